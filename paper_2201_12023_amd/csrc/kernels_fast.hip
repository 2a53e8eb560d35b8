// Table repack for the register/LDS recurrence kernel and its instances for up to 64 layers
// (the kernel itself: fast_kernel.hpp).
#include "fast_kernel.hpp"

namespace alpa {

__global__ void repack_fast_kernel(const int32_t *__restrict__ table, int K, int S, int KP,
                                   int32_t *__restrict__ recs)
{
    // one thread per (s, q, hb, column pair j): the pair record of last layers 2j and 2j+1
    const int NHB = KP / 8, NP = fast_pairs_per_row(K);
    const long long total = (long long)K * S * NHB * NP;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const int j = (int)(e % NP);
        long long r = e / NP;
        const int hb = (int)(r % NHB); r /= NHB;
        const int q = (int)(r % S);
        const int s = (int)(r / S);
        int32_t *rec = recs + e * PAIR_INTS;
        int32_t mn2 = DEV_INF, mx2 = -1;
        for (int half = 0; half < 2; ++half) {
            const int i = 2 * j + half;
            int32_t mn = DEV_INF, mx = -1;
            for (int u = 0; u < 8; ++u) {
                const int k = 8 * hb + u;
                int32_t v = DEV_INF;
                if (i < K && k <= i && k < K) {
                    const int32_t t = table[(((long long)s * K + k) * K + i) * S + q];
                    if (t != INF_I32) v = t;
                }
                rec[8 * half + u] = v;
                if (v < DEV_INF) { mn = min(mn, v); mx = max(mx, v); }
            }
            rec[18 + half] = (mx < 0) ? DEV_INF : mx;
            rec[20 + half] = mn;
            mn2 = min(mn2, mn);
            mx2 = max(mx2, mx);
        }
        rec[16] = mn2;
        rec[17] = (mx2 < 0) ? DEV_INF : mx2;
    }
}

// Second pass of the repack.  For every (q, half-block, group j of 8 columns (see end_group_cols), s) the minimum of
// t_intra over the half-block's first layers and all last layers >= 8j: a candidate below it
// finds nothing in column 8j or any later one, so the column loops of that (s, q, half-block)
// can stop there.  Layout g[q][hb][j][s - 1] with the s axis padded to SW = 64 (128 for more
// than 64 layers on more than 64 devices; stage counts exceed neither): the kernel reads it
// with lane = (s - 1) % 64.  Beyond 64 layers a group is KP / 8 columns wide.
__global__ void repack_group_min_kernel(int K, int S, int KP, int SW, const int32_t *__restrict__ recs,
                                        int32_t *__restrict__ g)
{
    const int NHB = KP / 8;
    const int total = S * NHB * SW;                    // one thread per (q, hb, s - 1)
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        const int s1 = e % SW;
        const int hb = (e / SW) % NHB;
        const int q = e / (SW * NHB);
        const int GW = end_group_cols(KP);
        int32_t run = DEV_INF;                         // no entry: alive for no candidate (the
                                                       // kernel clamps candidates below DEV_INF)
        for (int j = END_GROUPS - 1; j >= 0; --j) {
            if (s1 < K)
                for (int i = min(K, GW * j + GW) - 1; i >= GW * j; --i)    // the half-column's min
                    run = min(run, recs[((((long long)s1 * S + q) * NHB + hb) * fast_pairs_per_row(K) +
                                         (i >> 1)) * PAIR_INTS + 20 + (i & 1)]);
            g[((q * NHB + hb) * END_GROUPS + j) * SW + s1] = run;
        }
    }
}

// the records past the last column, which the loads that run ahead may touch: +infinity
__global__ void repack_padding_kernel(int32_t *__restrict__ p, int n)
{
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < n; x += gridDim.x * blockDim.x)
        p[x] = DEV_INF;
}

hipError_t launch_repack_fast(hipStream_t st, const int32_t *table, int K, int D, int S, int KP,
                              int32_t *recs, int32_t *group_min)
{
    const size_t real_ints = (size_t)K * S * (KP / 8) * fast_pairs_per_row(K) * PAIR_INTS;
    hipLaunchKernelGGL(repack_padding_kernel, dim3(8), dim3(256), 0, st, recs + real_ints,
                       (int)(fast_table_ints(K, S) - real_ints));
    long long total = (long long)K * S * (KP / 8) * fast_pairs_per_row(K);
    int grid = (int)((total + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(repack_fast_kernel, dim3(grid), dim3(256), 0, st, table, K, S, KP, recs);
    const int SW = fast_group_min_stages(K, D);
    const int n_chains = S * (KP / 8) * SW;
    hipLaunchKernelGGL(repack_group_min_kernel, dim3((n_chains + 63) / 64), dim3(64), 0, st, K, S,
                       KP, SW, recs, group_min);
    return hipGetLastError();
}

// stage counts the early-stop table spans (the kernel's SW)
int fast_group_min_stages(int K, int D) { return (K > 64 && D > WAVE) ? 2 * WAVE : WAVE; }

size_t fast_group_min_ints(int K, int D, int S)
{
    return (size_t)S * ((K + 15) / 16 * 2) * END_GROUPS * fast_group_min_stages(K, D);
}

size_t fast_table_ints(int K, int S)
{
    const int KP = 16 * ((K + 15) / 16);
    // the rows, and 64 pair records of padding
    return ((size_t)K * S * (KP / 8) * fast_pairs_per_row(K) + 64) * (size_t)PAIR_INTS;
}

// nc = candidates per workgroup (1 or 2; meshes of more than 64 devices: always one, in the
// two-window form); grid = persistent workgroups
hipError_t launch_recurrence_fast(hipStream_t st, const FastArgs &a, int mode, int nc, int grid)
{
    switch ((a.p.K + 15) / 16) {
    case 1: return launch_nwk<1>(st, a, mode, nc, grid);
    case 2: return launch_nwk<2>(st, a, mode, nc, grid);
    case 3: return launch_nwk<3>(st, a, mode, nc, grid);
    case 4: return launch_nwk<4>(st, a, mode, nc, grid);
    default: return launch_recurrence_fast_deep(st, a, mode, nc, grid);   // 65-128 layers
    }
}

// Resident workgroups of the batch-mode kernel per compute unit for nc candidates per
// workgroup, from the runtime's occupancy calculator.
int fast_kernel_blocks_per_cu(int K, int nc)
{
#define ALPA_BPC(NWK_) (nc == 2 ? blocks_per_cu<NWK_, 2>() : blocks_per_cu<NWK_, 1>())
    switch ((K + 15) / 16) {
    case 1: return ALPA_BPC(1);
    case 2: return ALPA_BPC(2);
    case 3: return ALPA_BPC(3);
    case 4: return ALPA_BPC(4);
    default: return fast_kernel_blocks_per_cu_deep(K, nc);
    }
#undef ALPA_BPC
}

}  // namespace alpa
