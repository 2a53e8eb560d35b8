// Construction of the stage-latency table on the device (Sec. 5.2, the paragraph that defines
// t_intra, Eq. 5, and the intra-op loop nest of Alg. 1): for every stage (k..i), submesh shape
// q and number s of stages from this one to the last, the lowest latency t_l among the profiled
// options whose memory fits, mem_stage + s * mem_act <= mem_device, else +infinity.
//
// One thread per (k, i, q).  All figures are non-negative (checked on the host), so an option
// fits exactly for s <= s_fit = floor((mem_device - mem_stage) / mem_act) (every s if mem_act
// is 0, none if mem_stage alone is too large); the thread keeps (t_l, s_fit) of its options in
// LDS and then emits one value per s.  Consecutive threads are consecutive (i, q), which is the
// fastest-varying part of the table's [s-1][k][i][q] layout, so each of the K rounds of stores
// is contiguous across the block.  HBM-bound on those stores: 4 K^3 S bytes out,
// 20 K^2 S O bytes in.
#include "internal.hpp"

namespace alpa {

constexpr int TABLE_BLOCK = 128;

__global__ __launch_bounds__(TABLE_BLOCK) void build_table_kernel(
    const int32_t *__restrict__ t_l, const int64_t *__restrict__ mem_stage,
    const int64_t *__restrict__ mem_act, int K, int S, int O, int64_t mem_device,
    int32_t *__restrict__ table, int32_t *__restrict__ max_finite)
{
    extern __shared__ int32_t opt[];                 // [O][TABLE_BLOCK] latency, then s_fit
    int32_t *opt_t = opt;
    int32_t *opt_s = opt + O * TABLE_BLOCK;
    const int tid = threadIdx.x;
    const long long n_entries = (long long)K * K * S;
    const long long e = (long long)blockIdx.x * TABLE_BLOCK + tid;
    const bool in = e < n_entries;
    int k = 0, i = 0;
    if (in) {
        const long long r = e / S;
        i = (int)(r % K);
        k = (int)(r / K);
    }
    const bool used = in && i >= k;
    for (int o = 0; o < O; ++o) {
        int32_t t = INF_I32, sf = 0;
        if (used) {
            const long long x = e * O + o;
            t = t_l[x];
            const int64_t ms = mem_stage[x], ma = mem_act[x];
            if (ms <= mem_device) {
                const int64_t room = mem_device - ms;
                sf = (ma == 0 || room / ma >= K) ? K : (int32_t)(room / ma);
            }
        }
        opt_t[o * TABLE_BLOCK + tid] = t;
        opt_s[o * TABLE_BLOCK + tid] = sf;
    }
    // own slots only: no barrier needed
    int32_t mx = -1;
    const long long slice = n_entries;               // entries per s
    for (int s = 1; s <= K; ++s) {
        int32_t m = INF_I32;
        for (int o = 0; o < O; ++o) {
            const int32_t t = opt_t[o * TABLE_BLOCK + tid];
            const int32_t sf = opt_s[o * TABLE_BLOCK + tid];
            m = (s <= sf && t < m) ? t : m;
        }
        if (in) table[(long long)(s - 1) * slice + e] = m;
        if (m != INF_I32 && m > mx) mx = m;
    }
    // largest finite entry of the table (for the range proof and the sort's key width)
    mx = max(mx, dpp_mov<0xB1>(mx));
    mx = max(mx, dpp_mov<0x4E>(mx));
    mx = max(mx, dpp_mov<0x141>(mx));
    mx = max(mx, dpp_mov<0x140>(mx));
    mx = max(mx, swz_xor16(mx));
    mx = max(mx, xor32(mx));
    if ((tid & (WAVE - 1)) == 0 && mx >= 0) atomicMax(max_finite, mx);
}

// "Equal layer" variant of the ablation study (Sec. 8.3): every stage of a plan has the same
// number of layers.  With s stages from first layer k to the end that number is (K - k) / s, so
// the restriction is a mask on the table: entry (s, k, i) stays iff s divides K - k and the
// stage k..i has exactly (K - k) / s layers.
__global__ void equal_layer_mask_kernel(int32_t *__restrict__ table, int K, int S)
{
    const long long total = (long long)K * K * K * S;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        long long r = e / S;
        const int i = (int)(r % K); r /= K;
        const int k = (int)(r % K);
        const int s = (int)(r / K) + 1;
        const int rest = K - k;
        const bool keep = rest % s == 0 && i - k + 1 == rest / s;
        if (!keep) table[e] = INF_I32;
    }
}

hipError_t launch_equal_layer_mask(hipStream_t st, int32_t *table, int K, int S)
{
    const long long total = (long long)K * K * K * S;
    int grid = (int)std::min<long long>((total + 255) / 256, 8192);
    hipLaunchKernelGGL(equal_layer_mask_kernel, dim3(grid), dim3(256), 0, st, table, K, S);
    return hipGetLastError();
}

__global__ void set_i32_kernel(int32_t *p, int32_t v)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

// Range of the part of a caller's table that the method reads (last layer >= first layer):
// out[0] = smallest entry (a negative one is an argument error), out[1] = largest finite entry
// (-1 if none; for the overflow proof and the sort's key width).  HBM-bound: 4 bytes per entry.
__global__ __launch_bounds__(256) void table_range_kernel(const int32_t *__restrict__ table, int K,
                                                          int S, int32_t *__restrict__ out)
{
    // one block per (s, first layer k): its used entries, last layers k..K-1, are contiguous
    const int k = blockIdx.x % K;
    const int32_t *row = table + (size_t)blockIdx.x * K * S;
    int32_t mn = INF_I32, mx = -1;
    for (int x = k * S + threadIdx.x; x < K * S; x += blockDim.x) {
        const int32_t t = row[x];
        mn = min(mn, t);
        if (t != INF_I32) mx = max(mx, t);
    }
    mn = wave_min_i32(mn);
    mx = -wave_min_i32(-mx);
    if ((threadIdx.x & (WAVE - 1)) == 0) {
        atomicMin(&out[0], mn);
        atomicMax(&out[1], mx);
    }
}

hipError_t launch_table_range(hipStream_t st, const int32_t *table, int K, int S, int32_t *out)
{
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(WAVE), 0, st, out + 0, INF_I32);
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(WAVE), 0, st, out + 1, -1);
    hipLaunchKernelGGL(table_range_kernel, dim3(K * K), dim3(256), 0, st, table, K, S, out);
    return hipGetLastError();
}

hipError_t launch_build_table(hipStream_t st, const int32_t *t_l, const int64_t *mem_stage,
                              const int64_t *mem_act, int K, int S, int O, int64_t mem_device,
                              int32_t *table, int32_t *max_finite)
{
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(WAVE), 0, st, max_finite, -1);
    const long long n_entries = (long long)K * K * S;
    const int grid = (int)((n_entries + TABLE_BLOCK - 1) / TABLE_BLOCK);
    const size_t lds = (size_t)O * TABLE_BLOCK * 2 * sizeof(int32_t);
    hipLaunchKernelGGL(build_table_kernel, dim3(grid), dim3(TABLE_BLOCK), lds, st, t_l, mem_stage,
                       mem_act, K, S, O, mem_device, table, max_finite);
    return hipGetLastError();
}

}  // namespace alpa
