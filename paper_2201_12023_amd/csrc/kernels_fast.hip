// Register/LDS recurrence kernel for K <= 64 layers and N*M <= 64 devices (Eq. 3).
//
// Mapping: one 64-lane wave evaluates one t_max candidate.  Lane l owns device count
// d = l + 1; the accumulators F(s, k, .) for ALL first layers k of the current s live in
// VGPRs (one register per k), the previous layer F(s-1, ., .) lives in LDS (one row of 64
// lanes per first layer).  For a fixed (last layer i, shape q) the operand
// F(s-1, i+1, d - a_q) is one lane-shifted LDS row read that is reused for every first
// layer k <= i, and t_intra(k..i, q, s) is the same for all lanes, so it is fetched with
// scalar loads and used as the scalar operand of the add: a cell-update costs one v_add
// and one v_min.  The filter t_intra <= t_max is wave-uniform; it is resolved per block of
// 16 first layers from that block's precomputed min / max (skip, take unfiltered, or
// select per entry).  Infinite entries need no filter: DEV_INF + anything >= DEV_INF and
// the accumulators start at DEV_INF.
//
// Table layout (built once per handle by repack_fast_kernel):
//   t_fast [s-1][i][q][kp]   kp = 0..KP-1 (KP = 16 * ceil(K/16)), first layer kp (0-based),
//                            last layer i (0-based); DEV_INF where kp > i, kp >= K or the
//                            entry is +infinity;
//   blk_mm [s-1][i][q][b][2] b = 0..3: {min over the block's entries, max over its finite
//                            entries (-1 if none)} for first layers 16b..16b+15.
#include "internal.hpp"

namespace alpa {

typedef const __attribute__((address_space(4))) int32_t *cptr_t;   // scalar-load path

__global__ void repack_fast_kernel(const int32_t *__restrict__ table, int K, int S, int KP,
                                   int32_t *__restrict__ t_fast, int32_t *__restrict__ blk_mm)
{
    // one thread per (s, i, q, b): fills 16 entries and their summary
    const long long total = (long long)K * K * S * 4;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int b = (int)(e & 3);
        long long r = e >> 2;
        const int q = (int)(r % S); r /= S;
        const int i = (int)(r % K);
        const int s = (int)(r / K);
        int32_t mn = DEV_INF, mx = -1;
        if (16 * b < KP) {
            int32_t *dst = t_fast + ((((long long)s * K + i) * S + q) * KP + 16 * b);
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
        int32_t *mm = blk_mm + ((((long long)s * K + i) * S + q) * 4 + b) * 2;
        mm[0] = mn;
        mm[1] = mx;
    }
}

template <int U>
__device__ __forceinline__ void relax16(int32_t (&acc)[64], cptr_t tp, int32_t G)
{
    int32_t t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = tp[u];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[U + u] = min(acc[U + u], t[u] + G);
}

template <int U>
__device__ __forceinline__ void relax16_filtered(int32_t (&acc)[64], cptr_t tp, int32_t G, int32_t c)
{
    int32_t t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = tp[u];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int32_t tu = (t[u] <= c) ? t[u] : DEV_INF;
        acc[U + u] = min(acc[U + u], tu + G);
    }
}

template <int U>
__device__ __forceinline__ void block_step(int32_t (&acc)[64], cptr_t tp, cptr_t mm, int32_t G,
                                           int32_t c, unsigned &n_blocks)
{
    const int32_t mn = mm[(U / 16) * 2 + 0], mx = mm[(U / 16) * 2 + 1];
    if (mn > c) return;                       // nothing in the block passes the filter
    ++n_blocks;
    if (mx <= c) relax16<U>(acc, tp + U, G);
    else relax16_filtered<U>(acc, tp + U, G, c);
}

__device__ bool can_skip_fast(const int64_t *chunk_min, int j, int32_t c, int B, int lane)
{
    const int g = j / PRUNE_CHUNK;
    int64_t m = INF_I64;
    for (int x = lane; x < g; x += WAVE)
        m = min64(m, __atomic_load_n(&chunk_min[x], __ATOMIC_RELAXED));
    m = wave_min_i64(m);
    return m != INF_I64 && (int64_t)B * (int64_t)c >= m;
}

// NB = number of 16-wide first-layer blocks (ceil(K / 16)); COUNT = tally executed blocks.
template <int NB, bool COUNT>
__global__ __launch_bounds__(WAVE) void recurrence_fast_kernel(
    Problem p, const int32_t *__restrict__ t_fast_g, const int32_t *__restrict__ blk_mm_g,
    const int32_t *__restrict__ sizes_g, const int32_t *__restrict__ cand, SolveState *state,
    int64_t *chunk_min, int prune, int descending, int32_t *__restrict__ Fmin,
    int32_t *__restrict__ Sbest)
{
    constexpr int KP = NB * 16;
    extern __shared__ int32_t Fprev[];                 // [K][64]
    const int lane = threadIdx.x;
    const int K = p.K, D = p.D, S = p.S;
    const cptr_t t_fast = (cptr_t)t_fast_g;
    const cptr_t blk_mm = (cptr_t)blk_mm_g;
    const cptr_t sizes = (cptr_t)sizes_g;
    const int n = __builtin_amdgcn_readfirstlane(state->n_cand);
    unsigned long long n_blocks_total = 0;

    for (;;) {
        // Every lane issues the atomic (lane 0 adds 1, the others 0) and lane 0's return
        // value is the ticket.  No branch on the lane id may appear in this loop: such a
        // branch is loop-invariant, the compiler splits the loop on it, and the lanes of
        // one wave then run the persistent loop out of step with each other.
        const int tk = __builtin_amdgcn_readfirstlane(
            atomicAdd(&state->ticket, lane == 0 ? 1 : 0));
        if (tk >= n) break;                            // the wave's only exit
        const int j = descending ? (n - 1 - tk) : tk;
        const int32_t c = __builtin_amdgcn_readfirstlane(cand[j]);
        if (prune && __builtin_amdgcn_readfirstlane((int)can_skip_fast(chunk_min, j, c, p.B, lane))) {
            Fmin[j] = DEV_INF;                         // all lanes, same value
            Sbest[j] = -1;
            continue;
        }
        int32_t best = DEV_INF, sbest = 0;
        unsigned n_blocks = 0;
        for (int s = 1; s <= p.Smax; ++s) {
            int32_t acc[64];
#pragma unroll
            for (int u = 0; u < 64; ++u) acc[u] = DEV_INF;
            const int i_lo = (s == 1) ? K - 1 : 0;     // 0-based last layer
            const int i_hi = K - s;                    // at least s-1 layers must remain
            for (int i = i_lo; i <= i_hi; ++i) {
                for (int q = 0; q < S; ++q) {
                    const int a = sizes[q];
                    if (a + s - 1 > D) continue;       // fewer than s-1 devices would remain
                    int32_t G;
                    if (s == 1) {
                        G = (lane + 1 == a) ? 0 : DEV_INF;          // F(0, K+1, 0) = 0
                    } else {
                        const int src = max(lane - a, 0);
                        const int32_t f = Fprev[(i + 1) * WAVE + src];   // F(s-1, i+1, d-a)
                        G = (lane >= a) ? f : DEV_INF;
                    }
                    const size_t col = ((size_t)(s - 1) * K + i) * S + q;
                    const cptr_t tp = t_fast + col * KP;
                    const cptr_t mm = blk_mm + col * 8;
                    block_step<0>(acc, tp, mm, G, c, n_blocks);
                    if (NB > 1 && i >= 16) block_step<16>(acc, tp, mm, G, c, n_blocks);
                    if (NB > 2 && i >= 32) block_step<32>(acc, tp, mm, G, c, n_blocks);
                    if (NB > 3 && i >= 48) block_step<48>(acc, tp, mm, G, c, n_blocks);
                }
            }
            // F(s, ., .) becomes the previous layer; row 0 is never an operand
#pragma unroll
            for (int u = 1; u < KP; ++u)
                if (u < K) Fprev[u * WAVE + lane] = acc[u];
            if (acc[0] < best) { best = acc[0]; sbest = s; }       // lowest s on ties
        }
        // lane D-1 holds F(s, first layer, all devices)
        const int32_t bestD = __builtin_amdgcn_readlane(best, D - 1);
        const int32_t sD = __builtin_amdgcn_readlane(sbest, D - 1);
        Fmin[j] = bestD;                               // all lanes, same value
        Sbest[j] = bestD >= DEV_INF ? 0 : sD;
        if (prune && bestD < DEV_INF)                  // uniform; the minimum is idempotent
            atomicMin((long long *)&chunk_min[j / PRUNE_CHUNK],
                      (long long)bestD + (long long)(p.B - 1) * (long long)c);
        if (COUNT) n_blocks_total += n_blocks;
    }
    if (COUNT && lane == 0) atomicAdd(&state->wave_relax, n_blocks_total * 16ull);
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

template <int NB>
static hipError_t launch_nb(hipStream_t st, const Problem &p, const int32_t *t_fast,
                            const int32_t *blk_mm, const int32_t *sizes, const int32_t *cand,
                            SolveState *state, int64_t *chunk_min, int prune, int count_work,
                            int descending, int32_t *Fmin, int32_t *Sbest, int grid)
{
    const size_t lds = (size_t)p.K * WAVE * sizeof(int32_t);
    if (count_work)
        hipLaunchKernelGGL((recurrence_fast_kernel<NB, true>), dim3(grid), dim3(WAVE), lds, st, p,
                           t_fast, blk_mm, sizes, cand, state, chunk_min, prune, descending, Fmin,
                           Sbest);
    else
        hipLaunchKernelGGL((recurrence_fast_kernel<NB, false>), dim3(grid), dim3(WAVE), lds, st, p,
                           t_fast, blk_mm, sizes, cand, state, chunk_min, prune, descending, Fmin,
                           Sbest);
    return hipGetLastError();
}

hipError_t launch_recurrence_fast(hipStream_t st, const Problem &p, const int32_t *t_fast,
                                  const int32_t *blk_mm, const int32_t *sizes, const int32_t *cand,
                                  SolveState *state, int64_t *chunk_min, int prune, int count_work,
                                  int descending, int32_t *Fmin, int32_t *Sbest, int grid)
{
    const int NB = (p.K + 15) / 16;
    switch (NB) {
    case 1: return launch_nb<1>(st, p, t_fast, blk_mm, sizes, cand, state, chunk_min, prune,
                                count_work, descending, Fmin, Sbest, grid);
    case 2: return launch_nb<2>(st, p, t_fast, blk_mm, sizes, cand, state, chunk_min, prune,
                                count_work, descending, Fmin, Sbest, grid);
    case 3: return launch_nb<3>(st, p, t_fast, blk_mm, sizes, cand, state, chunk_min, prune,
                                count_work, descending, Fmin, Sbest, grid);
    case 4: return launch_nb<4>(st, p, t_fast, blk_mm, sizes, cand, state, chunk_min, prune,
                                count_work, descending, Fmin, Sbest, grid);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace alpa

namespace alpa {

// Resident workgroups (= waves) of the recurrence kernel per compute unit, from the
// runtime's occupancy calculator (LDS is the limiter: K rows of 64 int32 per wave).
int fast_kernel_blocks_per_cu(int K)
{
    const size_t lds = (size_t)K * WAVE * sizeof(int32_t);
    int nb = 0;
    hipError_t e;
    switch ((K + 15) / 16) {
    case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, recurrence_fast_kernel<1, false>, WAVE, lds); break;
    case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, recurrence_fast_kernel<2, false>, WAVE, lds); break;
    case 3: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, recurrence_fast_kernel<3, false>, WAVE, lds); break;
    default: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, recurrence_fast_kernel<4, false>, WAVE, lds); break;
    }
    if (e != hipSuccess) return 0;
    return nb;
}

}  // namespace alpa
