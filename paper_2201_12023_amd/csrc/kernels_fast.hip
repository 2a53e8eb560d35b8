// Register/LDS recurrence kernel for K <= 64 layers and N*M <= 64 devices (Eq. 3).
//
// Mapping.  One workgroup evaluates one t_max candidate at a time (persistent workgroups
// draw candidates from a ticket counter).  Lane l of every wave owns device count
// d = l + 1.  The first layers k are cut into blocks of 16; wave (wk, wi) of the
// workgroup owns block wk and keeps its 16 accumulators F(s, k, .) in VGPRs; with WI > 1
// the (last layer) columns are dealt round-robin over the wi and the partial minima are
// merged through LDS.  The previous layer F(s-1, ., .) lives in LDS, one row of 64 lanes
// per first layer.  For a fixed (last layer i, shape q) the operand F(s-1, i+1, d - a_q)
// is one lane-shifted LDS row read, reused for the 16 first layers of the block, and
// t_intra(k..i, q, s) is the same for all lanes: it is fetched with scalar loads and used
// as the scalar operand of the add, so a cell-update costs one v_add and one v_min.  The
// filter t_intra <= t_max is wave-uniform; it is resolved per block from the block's
// precomputed min / max (skip, take unfiltered, or select per entry).  Infinite entries
// need no filter: DEV_INF + anything >= DEV_INF and accumulators start at DEV_INF.
// Lanes with d <= a_q are switched off for the whole column loop of shape q.
//
// Table layout (built once per handle by repack_fast_kernel):
//   t_fast [s-1][q][i][kp]   kp = 0..KP-1 (KP = 16 * ceil(K/16)) = first layer (0-based),
//                            i = last layer (0-based); DEV_INF where kp > i, kp >= K or
//                            the entry is +infinity;
//   blk_mm [s-1][q][i][b][2] b = 0..3: {min over the block's entries, max over its finite
//                            entries (-1 if none)} for first layers 16b..16b+15.
#include "internal.hpp"

namespace alpa {

typedef const __attribute__((address_space(4))) int32_t *cptr_t;   // scalar-load path

__global__ void repack_fast_kernel(const int32_t *__restrict__ table, int K, int S, int KP,
                                   int32_t *__restrict__ t_fast, int32_t *__restrict__ blk_mm)
{
    // one thread per (s, q, i, b): fills 16 entries and their summary
    const long long total = (long long)K * S * K * 4;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int b = (int)(e & 3);
        long long r = e >> 2;
        const int i = (int)(r % K); r /= K;
        const int q = (int)(r % S);
        const int s = (int)(r / S);
        const long long col = ((long long)s * S + q) * K + i;
        int32_t mn = DEV_INF, mx = -1;
        if (16 * b < KP) {
            int32_t *dst = t_fast + col * KP + 16 * b;
            for (int u = 0; u < 16; ++u) {
                const int k = 16 * b + u;
                int32_t v = DEV_INF;
                if (k <= i && k < K) {
                    const int32_t t = table[(((long long)s * K + k) * K + i) * S + q];
                    if (t != INF_I32) v = t;
                }
                dst[u] = v;
                if (v < DEV_INF) { mn = min(mn, v); mx = max(mx, v); }
            }
        }
        int32_t *mm = blk_mm + (col * 4 + b) * 2;
        mm[0] = mn;
        mm[1] = mx;
    }
}

// One (last layer, shape) column against the 16 first layers of this wave's block.
template <bool COUNT>
__device__ __forceinline__ void column(int32_t (&acc)[16], cptr_t tp, cptr_t mm, int32_t G,
                                       int32_t c, unsigned &n_blocks)
{
    const int32_t mn = mm[0], mx = mm[1];
    if (mn > c) return;                       // nothing in the block passes the filter
    if (COUNT) ++n_blocks;
    int32_t t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = tp[u];
    if (mx > c) {                             // mixed block: filter entry by entry (scalar)
#pragma unroll
        for (int u = 0; u < 16; ++u) t[u] = (t[u] <= c) ? t[u] : DEV_INF;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u] = min(acc[u], t[u] + G);
}

// Lower-index evidence for the pruning rule (see recurrence_generic_kernel).
__device__ __forceinline__ bool can_skip_fast(const int64_t *chunk_min, int j, int32_t c, int B,
                                              int lane)
{
    const int g = j / PRUNE_CHUNK;
    int64_t m = INF_I64;
    for (int x = lane; x < g; x += WAVE)
        m = min64(m, __atomic_load_n(&chunk_min[x], __ATOMIC_RELAXED));
    m = wave_min_i64(m);
    return m != INF_I64 && (int64_t)B * (int64_t)c >= m;
}

// NWK = waves along the first-layer axis (= ceil(K / 16)); WI = waves along the column
// axis; DUMP = also store every layer to F_all (plan recovery); COUNT = tally executed
// blocks.  Fmin / Sbest have a spare slot at index dummy_idx for the waves that do not
// own the result.
template <int NWK, int WI, bool DUMP, bool COUNT>
__global__ __launch_bounds__(WAVE * NWK * WI) void recurrence_fast_kernel(
    Problem p, const int32_t *__restrict__ t_fast_g, const int32_t *__restrict__ blk_mm_g,
    const int32_t *__restrict__ sizes_g, const int32_t *__restrict__ cand,
    const int32_t *__restrict__ n_cand_p, int32_t *ticket, unsigned long long *wave_relax,
    int64_t *chunk_min, int prune, int descending, int32_t *__restrict__ Fmin,
    int32_t *__restrict__ Sbest, int dummy_idx, int32_t *__restrict__ F_all)
{
    constexpr int NT = WAVE * NWK * WI;
    constexpr int KP = NWK * 16;
    extern __shared__ int32_t lds[];                   // Fprev [KP][64] (+ Fnext [KP][64])
    __shared__ int32_t sh_tk[NT];
    __shared__ int32_t sh_skip[NWK * WI];
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wid % NWK, wi = wid / NWK;
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    const cptr_t t_fast = (cptr_t)t_fast_g;
    const cptr_t blk_mm = (cptr_t)blk_mm_g;
    const cptr_t sizes = (cptr_t)sizes_g;
    int32_t *Fprev = lds;
    int32_t *Fnext = lds + KP * WAVE;
    const int n = __builtin_amdgcn_readfirstlane(*n_cand_p);
    unsigned long long n_blocks_total = 0;

    for (;;) {
        // Every thread issues the atomic (thread 0 adds 1, the others 0) and all read thread
        // 0's return value.  No branch on the thread id may appear in this loop: it would be
        // loop-invariant, the compiler splits the loop on it, and the lanes of one wave then
        // run the persistent loop out of step with each other.
        sh_tk[tid] = atomicAdd(ticket, tid == 0 ? 1 : 0);
        __syncthreads();
        const int tk = __builtin_amdgcn_readfirstlane(sh_tk[0]);
        __syncthreads();
        if (tk >= n) break;                            // the workgroup's only exit
        const int j = descending ? (n - 1 - tk) : tk;
        const int32_t c = __builtin_amdgcn_readfirstlane(cand[j]);
        if (prune) {
            // wave 0's reading of the published minima decides for the whole workgroup
            sh_skip[wid] = can_skip_fast(chunk_min, j, c, p.B, lane) ? 1 : 0;
            __syncthreads();
            const int skip = __builtin_amdgcn_readfirstlane(sh_skip[0]);
            __syncthreads();
            if (skip) {
                Fmin[j] = DEV_INF;                     // all threads, same value
                Sbest[j] = -1;
                continue;
            }
        }
        if (DUMP) {
            const int total = (p.Smax + 1) * LS;
            for (int x = tid; x < total; x += NT) F_all[x] = (x == (K + 1) * (D + 1)) ? 0 : DEV_INF;
            __syncthreads();
        }
        int32_t best = DEV_INF, sbest = 0;
        unsigned n_blocks = 0;
        for (int s = 1; s <= p.Smax; ++s) {
            int32_t acc[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc[u] = DEV_INF;
            const int i_lo = (s == 1) ? K - 1 : 0;     // 0-based last layer
            const int i_hi = K - s;                    // at least s-1 layers must remain
            const int i0 = max(i_lo, 16 * wk) + wi;    // columns with a first layer in this block
            if (WI > 1) {
                for (int x = tid; x < KP * WAVE; x += NT) Fnext[x] = DEV_INF;
            }
            for (int q = 0; q < S; ++q) {
                const int a = sizes[q];
                if (a + s - 1 > D) continue;           // fewer than s-1 devices would remain
                const size_t colq = ((size_t)(s - 1) * S + q) * K;
                if (s == 1) {
                    const int32_t G = (lane + 1 == a) ? 0 : DEV_INF;     // F(0, K+1, 0) = 0
                    for (int i = i0; i <= i_hi; i += WI)
                        column<COUNT>(acc, t_fast + (colq + i) * KP + 16 * wk,
                                      blk_mm + ((colq + i) * 4 + wk) * 2, G, c, n_blocks);
                } else {
                    const bool live = lane >= a;       // d - a_q >= 1
                    const int32_t *row = Fprev + (live ? lane - a : 0);
                    for (int i = i0; i <= i_hi; i += WI) {
                        const int32_t f = row[(i + 1) * WAVE];           // F(s-1, i+1, d-a)
                        const int32_t G = live ? f : DEV_INF;
                        column<COUNT>(acc, t_fast + (colq + i) * KP + 16 * wk,
                                      blk_mm + ((colq + i) * 4 + wk) * 2, G, c, n_blocks);
                    }
                }
            }
            __syncthreads();                           // every wave is done reading Fprev
            int32_t f1;
            if (WI == 1) {
#pragma unroll
                for (int u = 0; u < 16; ++u)           // rows 0 and >= K are never operands
                    Fprev[(16 * wk + u) * WAVE + lane] = acc[u];
                __syncthreads();
                f1 = acc[0];                           // F(s, first layer, .) in the wk = 0 wave
            } else {
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    atomicMin(&Fnext[(16 * wk + u) * WAVE + lane], acc[u]);
                __syncthreads();
                int32_t *tmp = Fprev; Fprev = Fnext; Fnext = tmp;
                f1 = Fprev[lane];                      // row 0 holds F(s, first layer, .)
            }
            if (f1 < best) { best = f1; sbest = s; }   // lowest s on ties
            if (DUMP) {
                int32_t *Fs = F_all + (size_t)s * LS;
                if (WI == 1) {
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int k = 16 * wk + u;
                        const bool in = lane < D;
                        if (k < K) Fs[(k + 1) * (D + 1) + (in ? lane + 1 : 0)] = in ? acc[u] : DEV_INF;
                    }
                } else {
                    // lanes beyond the mesh rewrite the row's d = 0 cell with infinity
                    // (a select, not a branch on the lane id: see the ticket comment)
                    for (int x = tid; x < K * WAVE; x += NT) {
                        const int k = x >> 6, l = x & (WAVE - 1);
                        const bool in = l < D;
                        Fs[(k + 1) * (D + 1) + (in ? l + 1 : 0)] = in ? Fprev[x] : DEV_INF;
                    }
                }
            }
        }
        // lane D-1 holds F(s, first layer, all devices); wave 0 owns the result
        const int32_t bestD = __builtin_amdgcn_readlane(best, D - 1);
        const int32_t sD = __builtin_amdgcn_readlane(sbest, D - 1);
        const bool owner = (wid == 0);
        const int slot = owner ? j : dummy_idx;
        Fmin[slot] = bestD;                            // all lanes, same value
        Sbest[slot] = bestD >= DEV_INF ? 0 : sD;
        if (prune) {                                   // uniform; the minimum is idempotent
            const long long T = (owner && bestD < DEV_INF)
                                    ? (long long)bestD + (long long)(p.B - 1) * (long long)c
                                    : (long long)INF_I64;
            atomicMin((long long *)&chunk_min[j / PRUNE_CHUNK], T);
        }
        if (COUNT) n_blocks_total += n_blocks;
        __syncthreads();                               // LDS is reused by the next candidate
    }
    if (COUNT) atomicAdd(wave_relax, lane == 0 ? n_blocks_total * 16ull : 0ull);
}

hipError_t launch_repack_fast(hipStream_t st, const int32_t *table, int K, int S, int KP,
                              int32_t *t_fast, int32_t *blk_mm)
{
    long long total = (long long)K * K * S * 4;
    int grid = (int)((total + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(repack_fast_kernel, dim3(grid), dim3(256), 0, st, table, K, S, KP, t_fast,
                       blk_mm);
    return hipGetLastError();
}

constexpr int PLAN_WI = 4;       // column-axis waves of the single-candidate (plan) run

template <int NWK, int WI, bool DUMP, bool COUNT>
static hipError_t launch_one(hipStream_t st, const FastArgs &a, int grid)
{
    const size_t lds = (size_t)NWK * 16 * WAVE * sizeof(int32_t) * (WI > 1 ? 2 : 1);
    hipLaunchKernelGGL((recurrence_fast_kernel<NWK, WI, DUMP, COUNT>), dim3(grid),
                       dim3(WAVE * NWK * WI), lds, st, a.p, a.t_fast, a.blk_mm, a.sizes, a.cand,
                       a.n_cand_p, a.ticket, a.wave_relax, a.chunk_min, a.prune, a.descending,
                       a.Fmin, a.Sbest, a.dummy_idx, a.F_all);
    return hipGetLastError();
}

template <int NWK>
static hipError_t launch_nwk(hipStream_t st, const FastArgs &a, int mode, int grid)
{
    switch (mode) {
    case FAST_MODE_PLAN: return launch_one<NWK, PLAN_WI, true, false>(st, a, grid);
    case FAST_MODE_COUNT: return launch_one<NWK, 1, false, true>(st, a, grid);
    default: return launch_one<NWK, 1, false, false>(st, a, grid);
    }
}

hipError_t launch_recurrence_fast(hipStream_t st, const FastArgs &a, int mode, int grid)
{
    switch ((a.p.K + 15) / 16) {
    case 1: return launch_nwk<1>(st, a, mode, grid);
    case 2: return launch_nwk<2>(st, a, mode, grid);
    case 3: return launch_nwk<3>(st, a, mode, grid);
    case 4: return launch_nwk<4>(st, a, mode, grid);
    default: return hipErrorInvalidValue;
    }
}

// Resident workgroups of the batch-mode kernel per compute unit, from the runtime's
// occupancy calculator.
int fast_kernel_blocks_per_cu(int K)
{
    const size_t lds = (size_t)((K + 15) / 16) * 16 * WAVE * sizeof(int32_t);
    int nb = 0;
    hipError_t e;
    switch ((K + 15) / 16) {
    case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &nb, recurrence_fast_kernel<1, 1, false, false>, WAVE * 1, lds); break;
    case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &nb, recurrence_fast_kernel<2, 1, false, false>, WAVE * 2, lds); break;
    case 3: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &nb, recurrence_fast_kernel<3, 1, false, false>, WAVE * 3, lds); break;
    default: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &nb, recurrence_fast_kernel<4, 1, false, false>, WAVE * 4, lds); break;
    }
    if (e != hipSuccess) return 0;
    return nb;
}

}  // namespace alpa
