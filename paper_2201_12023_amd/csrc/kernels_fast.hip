// Register/LDS recurrence kernel for K <= 64 layers and N*M <= 64 devices (Eq. 3).
//
// Mapping.  One workgroup evaluates one t_max candidate at a time (persistent workgroups
// draw candidates from a ticket counter).  Lane l of every wave owns device count
// d = l + 1.  The first layers k are cut into half-blocks of 8; a workgroup has NWK =
// ceil(K / 16) waves along that axis and wave w owns half-blocks w ("A") and 2*NWK-1-w
// ("B"): the triangular work (a column with last layer i only touches first layers <= i)
// is then the same for every wave.  The 16 accumulators F(s, k, .) of a wave live in VGPRs;
// with WI > 1 the (last layer) columns are dealt round-robin over WI wave groups and the
// partial minima are merged through LDS.  The previous layer F(s-1, ., .) lives in LDS, one
// row of 64 lanes per first layer.  For a fixed (last layer i, shape q) the operand
// F(s-1, i+1, d - a_q) is one lane-shifted LDS row read, reused for all first layers of the
// wave, and t_intra(k..i, q, s) is the same for all lanes: it is fetched with scalar loads
// and used as the scalar operand of the add, so a cell-update costs one v_add and one v_min.
// The filter t_intra <= t_max is wave-uniform; it is resolved per half-block from its
// precomputed min / max (skip, take unfiltered, or select per entry on the scalar unit).
// Infinite entries need no filter: DEV_INF + anything >= DEV_INF and accumulators start at
// DEV_INF.  Column loads (scalars and the LDS row) are issued one column ahead.
//
// Table layout (built once per handle by repack_fast_kernel): one record per column
// (s-1, q, i), columns in that order (i fastest); a record is KP/8 half-block entries of
// HB_INTS = 10 int32 (KP = 16 * ceil(K/16)):
//   {min, max over the finite t_intra of first layers 8hb..8hb+7 and last layer i
//    ({DEV_INF, DEV_INF} if there is none), then the 8 values themselves: DEV_INF where the
//    first layer is > i or >= K or the entry is +infinity}.
// The array is padded by a few records so that the one-column-ahead loads may run past the
// last column.
#include "internal.hpp"

namespace alpa {

typedef const __attribute__((address_space(4))) int32_t *cptr_t;   // scalar-load path

constexpr int HB_INTS = 10;

__global__ void repack_fast_kernel(const int32_t *__restrict__ table, int K, int S, int KP,
                                   int32_t *__restrict__ recs)
{
    // one thread per (s, q, i, hb)
    const int NHB = KP / 8;
    const long long total = (long long)K * S * K * NHB;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int hb = (int)(e % NHB);
        long long r = e / NHB;
        const int i = (int)(r % K); r /= K;
        const int q = (int)(r % S);
        const int s = (int)(r / S);
        int32_t *rec = recs + ((((long long)s * S + q) * K + i) * NHB + hb) * HB_INTS;
        int32_t mn = DEV_INF, mx = -1;
        for (int u = 0; u < 8; ++u) {
            const int k = 8 * hb + u;
            int32_t v = DEV_INF;
            if (k <= i && k < K) {
                const int32_t t = table[(((long long)s * K + k) * K + i) * S + q];
                if (t != INF_I32) v = t;
            }
            rec[2 + u] = v;
            if (v < DEV_INF) { mn = min(mn, v); mx = max(mx, v); }
        }
        rec[0] = mn;
        rec[1] = (mx < 0) ? DEV_INF : mx;
    }
}

// One half-block's share of a column, loaded one step ahead of its use.
struct HalfColumn {
    int32_t t[8];              // t_intra for 8 first layers (scalar registers)
    int32_t mn, mx;            // the half-block's min / max over finite entries
};

__device__ __forceinline__ void load_half(HalfColumn &h, cptr_t rec)
{
    h.mn = rec[0];
    h.mx = rec[1];
#pragma unroll
    for (int u = 0; u < 8; ++u) h.t[u] = rec[2 + u];
}

// Makes loaded values "used" here, so that the wait for them is placed before the next
// loads are issued (scalar loads return out of order: any later wait would also wait for
// the loads just issued).  The memory clobber keeps later loads below this point.
__device__ __forceinline__ void settle(const HalfColumn &h)
{
    asm volatile("" :: "s"(h.t[0]), "s"(h.t[1]), "s"(h.t[2]), "s"(h.t[3]), "s"(h.t[4]),
                       "s"(h.t[5]), "s"(h.t[6]), "s"(h.t[7]), "s"(h.mn), "s"(h.mx)
                 : "memory");
}
__device__ __forceinline__ void settle(const HalfColumn &h, int32_t f)
{
    asm volatile("" :: "s"(h.t[0]), "s"(h.t[1]), "s"(h.t[2]), "s"(h.t[3]), "s"(h.t[4]),
                       "s"(h.t[5]), "s"(h.t[6]), "s"(h.t[7]), "s"(h.mn), "s"(h.mx), "v"(f)
                 : "memory");
}
__device__ __forceinline__ void fence_loads() { asm volatile("" ::: "memory"); }

// Eight first layers against one column: unfiltered when every finite entry passes, skipped
// when none does, else filtered entry by entry on the scalar unit.
template <bool COUNT>
__device__ __forceinline__ void relax8(int32_t *acc, int32_t (&t)[8], int32_t mn, int32_t mx,
                                       int32_t G, int32_t c, unsigned &n_blocks)
{
    if (mn <= c) {                            // else nothing in the half-block passes
        if (mx > c) {
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = (t[u] <= c) ? t[u] : DEV_INF;
        }
        if (COUNT) ++n_blocks;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = min(acc[u], t[u] + G);
    }
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
    Problem p, const int32_t *__restrict__ recs_g, const int32_t *__restrict__ sizes_g, const int32_t *__restrict__ cand,
    const int32_t *__restrict__ n_cand_p, int32_t *ticket, unsigned long long *wave_relax,
    int64_t *chunk_min, int prune, int descending, int32_t *__restrict__ Fmin,
    int32_t *__restrict__ Sbest, int dummy_idx, int32_t *__restrict__ F_all)
{
    constexpr int NT = WAVE * NWK * WI;
    constexpr int KP = NWK * 16;
    extern __shared__ int32_t lds[];                   // Fprev [KP+WI][64] (+ Fnext, same size)
    __shared__ int32_t sh_tk[NT];
    __shared__ int32_t sh_skip[NWK * WI];
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wid % NWK, wi = wid / NWK;
    const int hbA = wk, hbB = 2 * NWK - 1 - wk;        // the wave's two half-blocks of 8 first layers
    const int rowA = 8 * hbA, rowB = 8 * hbB;
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    constexpr int REC = (KP / 8) * HB_INTS;            // int32 per column record
    const cptr_t recs = (cptr_t)recs_g;
    const cptr_t sizes = (cptr_t)sizes_g;
    int32_t *Fprev = lds;
    int32_t *Fnext = lds + (KP + WI) * WAVE;
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
            int32_t acc[16];                           // [0..7] half-block A, [8..15] half-block B
#pragma unroll
            for (int u = 0; u < 16; ++u) acc[u] = DEV_INF;
            const int i_lo = (s == 1) ? K - 1 : 0;     // 0-based last layer
            const int i_hi = K - s;                    // at least s-1 layers must remain
            const int i0 = max(i_lo, rowA) + wi;       // columns that reach half-block A
            if (WI > 1) {
                for (int x = tid; x < (KP + WI) * WAVE; x += NT) Fnext[x] = DEV_INF;
            }
            for (int q = 0; q < S; ++q) {
                const int a = sizes[q];
                if (a + s - 1 > D) continue;           // fewer than s-1 devices would remain
                if (i0 > i_hi) continue;
                constexpr int STEP = REC * WI;
                const cptr_t rec0 = recs + (((size_t)(s - 1) * S + q) * K + i0) * REC;   // column i0
                cptr_t pA = rec0 + hbA * HB_INTS, pB = rec0 + hbB * HB_INTS;
                const int ncol = (i_hi - i0) / WI + 1;         // columns of this wave
                HalfColumn hA, hB;
                if (s == 1) {
                    // F(0, K+1, 0) = 0 is the only finite operand: last layer K-1, d = a_q
                    const int32_t G = (lane + 1 == a) ? 0 : DEV_INF;
                    int i = i0;
                    for (int x = 0; x < ncol; ++x, pA += STEP, pB += STEP, i += WI) {
                        load_half(hA, pA);
                        load_half(hB, pB);
                        relax8<COUNT>(acc, hA.t, hA.mn, hA.mx, G, c, n_blocks);
                        if (i >= rowB) relax8<COUNT>(acc + 8, hB.t, hB.mn, hB.mx, G, c, n_blocks);
                    }
                    continue;
                }
                // Pipeline, one step ahead: while half-block A of a column is computed the
                // loads for its half-block B are in flight, and while B is computed the loads
                // for A of the next column (and that column's LDS row) are.  The loads after
                // the last column land in the padding and are dropped.
                const bool live = lane >= a;           // d - a_q >= 1
                const int32_t *frow = Fprev + (live ? lane - a : 0) + (i0 + 1) * WAVE;   // row i+1
                int32_t f = *frow;
                load_half(hA, pA);
                fence_loads();
                // columns that only reach half-block A, two per trip (hB serves as the
                // second buffer); an odd one is done without overlap
                const int n1 = max(0, min((rowB - i0 + WI - 1) / WI, ncol));
                for (int x = n1 >> 1; x > 0; --x) {
                    settle(hA, f);
                    frow += WAVE * WI;
                    int32_t f2 = *frow;
                    load_half(hB, pA + STEP);
                    fence_loads();
                    const int32_t G = live ? f : DEV_INF;
                    relax8<COUNT>(acc, hA.t, hA.mn, hA.mx, G, c, n_blocks);
                    settle(hB, f2);
                    frow += WAVE * WI;
                    f = *frow;
                    pA += 2 * STEP;
                    load_half(hA, pA);
                    fence_loads();
                    const int32_t G2 = live ? f2 : DEV_INF;
                    relax8<COUNT>(acc, hB.t, hB.mn, hB.mx, G2, c, n_blocks);
                }
                if (n1 & 1) {
                    const int32_t G = live ? f : DEV_INF;
                    relax8<COUNT>(acc, hA.t, hA.mn, hA.mx, G, c, n_blocks);
                    pA += STEP;
                    frow += WAVE * WI;
                    f = *frow;
                    load_half(hA, pA);
                    fence_loads();
                }
                // columns that reach both half-blocks
                pB += (size_t)n1 * STEP;
                for (int x = ncol - n1; x > 0; --x) {
                    settle(hA, f);
                    load_half(hB, pB);
                    fence_loads();
                    const int32_t G = live ? f : DEV_INF;
                    relax8<COUNT>(acc, hA.t, hA.mn, hA.mx, G, c, n_blocks);
                    settle(hB);
                    frow += WAVE * WI;
                    f = *frow;
                    pA += STEP;
                    pB += STEP;
                    load_half(hA, pA);
                    fence_loads();
                    relax8<COUNT>(acc + 8, hB.t, hB.mn, hB.mx, G, c, n_blocks);
                }
            }
            __syncthreads();                           // every wave is done reading Fprev
            int32_t f1;
            if (WI == 1) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {          // rows 0 and >= K are never operands
                    Fprev[(rowA + u) * WAVE + lane] = acc[u];
                    Fprev[(rowB + u) * WAVE + lane] = acc[8 + u];
                }
                __syncthreads();
                f1 = acc[0];                           // F(s, first layer, .) in wave 0 (half-block 0)
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    atomicMin(&Fnext[(rowA + u) * WAVE + lane], acc[u]);
                    atomicMin(&Fnext[(rowB + u) * WAVE + lane], acc[8 + u]);
                }
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
                        const int k = (u < 8 ? rowA : rowB - 8) + u;
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
    if (COUNT) atomicAdd(wave_relax, lane == 0 ? n_blocks_total * 8ull : 0ull);
}

hipError_t launch_repack_fast(hipStream_t st, const int32_t *table, int K, int S, int KP,
                              int32_t *recs)
{
    long long total = (long long)K * K * S * (KP / 8);
    int grid = (int)((total + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(repack_fast_kernel, dim3(grid), dim3(256), 0, st, table, K, S, KP, recs);
    return hipGetLastError();
}

size_t fast_table_ints(int K, int S)
{
    const int KP = 16 * ((K + 15) / 16);
    return ((size_t)K * S * K + 8) * (size_t)((KP / 8) * HB_INTS);     // 8 records of padding
}

constexpr int PLAN_WI = 4;       // column-axis waves of the single-candidate (plan) run

template <int NWK, int WI, bool DUMP, bool COUNT>
static hipError_t launch_one(hipStream_t st, const FastArgs &a, int grid)
{
    const size_t lds = (size_t)(NWK * 16 + WI) * WAVE * sizeof(int32_t) * (WI > 1 ? 2 : 1);
    hipLaunchKernelGGL((recurrence_fast_kernel<NWK, WI, DUMP, COUNT>), dim3(grid),
                       dim3(WAVE * NWK * WI), lds, st, a.p, a.recs, a.sizes, a.cand,
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
    const size_t lds = (size_t)(((K + 15) / 16) * 16 + 1) * WAVE * sizeof(int32_t);
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
