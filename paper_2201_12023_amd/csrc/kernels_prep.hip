// Candidate preparation on the device: the "SortedAndFilter(t_intra, epsilon)" step of
// Alg. 1.  Latencies are integer microseconds and epsilon is 1 us (Sec. 5.2, performance
// optimisation #1), so the step is: ascending order, duplicates removed.
//
// Kernels: gather of the table's values, a least-significant-digit radix sort (8-bit
// digits, one wave per slice, stable ranking inside a wave by ballot matching), adjacent
// -difference flags + scan + compaction, quantile pick, and rank lookup for the caller's
// own candidate order.
#include "internal.hpp"

namespace alpa {

constexpr int SORT_BLOCKS = SORT_SLICES;   // one wave each, contiguous slice per wave
constexpr int RADIX = SORT_RADIX;

// ---------------------------------------------------------------- gather

// One key per table entry with last layer >= first layer, at a fixed position, so that
// the number of keys is known on the host; +infinity becomes `inf_key` (largest finite
// value + 1) and is dropped again after the sort.
__global__ void gather_table_values_kernel(const int32_t *__restrict__ table, int K, int S,
                                           int32_t inf_key, int32_t *__restrict__ keys)
{
    const long long total = (long long)K * K * K * S;
    const int P = K * (K + 1) / 2;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        int q = (int)(e % S);
        long long r = e / S;
        int i = (int)(r % K); r /= K;
        int k = (int)(r % K);
        int s = (int)(r / K);
        if (i < k) continue;
        int tri = k * K - (k * (k - 1)) / 2 + (i - k);
        int32_t t = table[e];
        keys[((long long)s * P + tri) * S + q] = (t == INF_I32) ? inf_key : t;
    }
}

// ---------------------------------------------------------------- radix sort

__device__ __forceinline__ void slice_of(int n, int b, int &lo, int &hi)
{
    int per = (n + SORT_BLOCKS - 1) / SORT_BLOCKS;
    per = (per + WAVE - 1) / WAVE * WAVE;
    lo = min(n, b * per);
    hi = min(n, lo + per);
}

__global__ __launch_bounds__(WAVE) void radix_hist_kernel(const int32_t *__restrict__ keys, int n,
                                                          int shift, uint32_t *__restrict__ hist)
{
    __shared__ uint32_t cnt[RADIX];
    const int lane = threadIdx.x;
    for (int x = lane; x < RADIX; x += WAVE) cnt[x] = 0;
    __syncthreads();
    int lo, hi;
    slice_of(n, blockIdx.x, lo, hi);
    for (int j = lo + lane; j < hi; j += WAVE) {
        uint32_t dgt = ((uint32_t)keys[j] >> shift) & (RADIX - 1);
        atomicAdd(&cnt[dgt], 1u);
    }
    __syncthreads();
    for (int x = lane; x < RADIX; x += WAVE) hist[x * SORT_BLOCKS + blockIdx.x] = cnt[x];
}

// Exclusive scan of `len` uint32 values in place, one block of 1024 threads: every thread
// owns a contiguous segment.
__global__ __launch_bounds__(1024) void scan_u32_kernel(uint32_t *__restrict__ v, int len,
                                                        uint32_t *__restrict__ total_out)
{
    __shared__ uint32_t part[1024];
    const int t = threadIdx.x;
    const int L = (len + 1023) / 1024;
    const int lo = min(len, t * L), hi = min(len, lo + L);
    uint32_t s = 0;
    for (int j = lo; j < hi; ++j) s += v[j];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        uint32_t o = (t >= off) ? part[t - off] : 0u;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    uint32_t run = part[t] - s;
    for (int j = lo; j < hi; ++j) {
        uint32_t x = v[j];
        v[j] = run;
        run += x;
    }
    if (total_out && t == 1023) *total_out = part[1023];
}

// Offsets of one radix pass from the per-slice digit counts hist[digit][slice]: one block per
// digit scans its SORT_BLOCKS counts in place (exclusive) and leaves the digit's total in
// totals[digit]; digit_base_kernel then scans the 256 totals.
__global__ __launch_bounds__(SORT_BLOCKS) void digit_scan_kernel(uint32_t *__restrict__ hist,
                                                                 uint32_t *__restrict__ totals)
{
    __shared__ uint32_t part[SORT_BLOCKS];
    const int t = threadIdx.x;
    uint32_t *row = hist + blockIdx.x * SORT_BLOCKS;
    const uint32_t own = row[t];
    part[t] = own;
    __syncthreads();
    for (int off = 1; off < SORT_BLOCKS; off <<= 1) {
        const uint32_t o = (t >= off) ? part[t - off] : 0u;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    row[t] = part[t] - own;
    if (t == SORT_BLOCKS - 1) totals[blockIdx.x] = part[t];
}

__global__ __launch_bounds__(RADIX) void digit_base_kernel(uint32_t *__restrict__ totals)
{
    __shared__ uint32_t part[RADIX];
    const int t = threadIdx.x;
    const uint32_t own = totals[t];
    part[t] = own;
    __syncthreads();
    for (int off = 1; off < RADIX; off <<= 1) {
        const uint32_t o = (t >= off) ? part[t - off] : 0u;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    totals[t] = part[t] - own;
}

__global__ __launch_bounds__(WAVE) void radix_scatter_kernel(const int32_t *__restrict__ keys_in,
                                                             int32_t *__restrict__ keys_out, int n,
                                                             int shift,
                                                             const uint32_t *__restrict__ offs,
                                                             const uint32_t *__restrict__ digit_base)
{
    __shared__ uint32_t base[RADIX];
    const int lane = threadIdx.x;
    for (int x = lane; x < RADIX; x += WAVE)
        base[x] = digit_base[x] + offs[x * SORT_BLOCKS + blockIdx.x];
    __syncthreads();
    int lo, hi;
    slice_of(n, blockIdx.x, lo, hi);
    const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int j0 = lo; j0 < hi; j0 += WAVE) {
        const int j = j0 + lane;
        const bool valid = j < hi;
        const int32_t key = valid ? keys_in[j] : 0;
        const uint32_t dgt = ((uint32_t)key >> shift) & (RADIX - 1);
        uint64_t m = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (dgt >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            m &= bit ? bal : ~bal;
        }
        const uint32_t rank = (uint32_t)__popcll(m & lt);
        uint32_t pos = 0;
        if (valid) pos = base[dgt] + rank;
        __syncthreads();
        if (valid && rank == 0) base[dgt] += (uint32_t)__popcll(m);
        __syncthreads();
        if (valid) keys_out[pos] = key;
    }
}

// ---------------------------------------------------------------- dedup

constexpr int DEDUP_TILE = 1024 * 4;

__device__ __forceinline__ uint32_t head_flag(const int32_t *keys, int j, int n, int32_t drop_key)
{
    if (j >= n) return 0u;
    const int32_t x = keys[j];
    if (x == drop_key) return 0u;
    return (j == 0 || keys[j - 1] != x) ? 1u : 0u;
}

__global__ __launch_bounds__(1024) void dedup_count_kernel(const int32_t *__restrict__ keys, int n,
                                                           int32_t drop_key,
                                                           uint32_t *__restrict__ block_cnt)
{
    __shared__ uint32_t wsum[16];
    const int t = threadIdx.x;
    const int base = blockIdx.x * DEDUP_TILE + t * 4;
    uint32_t c = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) c += head_flag(keys, base + u, n, drop_key);
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);
    if ((t & 63) == 0) wsum[t >> 6] = c;
    __syncthreads();
    if (t == 0) {
        uint32_t s = 0;
        for (int w = 0; w < 16; ++w) s += wsum[w];
        block_cnt[blockIdx.x] = s;
    }
}

__global__ __launch_bounds__(1024) void dedup_write_kernel(const int32_t *__restrict__ keys, int n,
                                                           int32_t drop_key,
                                                           const uint32_t *__restrict__ block_off,
                                                           int32_t *__restrict__ unique)
{
    __shared__ uint32_t part[1024];
    const int t = threadIdx.x;
    const int base = blockIdx.x * DEDUP_TILE + t * 4;
    uint32_t f[4], c = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) { f[u] = head_flag(keys, base + u, n, drop_key); c += f[u]; }
    part[t] = c;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        uint32_t o = (t >= off) ? part[t - off] : 0u;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    uint32_t pos = block_off[blockIdx.x] + part[t] - c;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (f[u]) unique[pos++] = keys[base + u];
}

// ---------------------------------------------------------------- distinct values by bitmap
//
// SortedAndFilter of Alg. 1 for tables whose finite values are small integers (below
// DISTINCT_BITMAP_MAX, so that the bitmap fits a workgroup's 64 KiB of LDS): instead of sorting every entry, each finite entry sets one bit of a
// presence bitmap and the set bits are listed in order; the result is the same ascending list
// of distinct values.

__global__ void bitmap_clear_kernel(uint32_t *__restrict__ bm, int words)
{
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < words; x += gridDim.x * blockDim.x)
        bm[x] = 0u;
}

// Every block marks its share of the table in a bitmap of its own in LDS (most entries repeat
// values the block has already seen) and then merges the words it touched into the global one.
__global__ __launch_bounds__(1024) void bitmap_mark_kernel(const int32_t *__restrict__ table, int K,
                                                           int S, int words,
                                                           uint32_t *__restrict__ bm)
{
    extern __shared__ uint32_t lbm[];             // [words]
    for (int x = threadIdx.x; x < words; x += blockDim.x) lbm[x] = 0u;
    __syncthreads();
    const long long total = (long long)K * K * K * S;
    for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const long long r = e / S;
        const int i = (int)(r % K), k = (int)((r / K) % K);
        if (i < k) continue;
        const int32_t t = table[e];
        if (t == INF_I32) continue;
        const uint32_t bit = 1u << (t & 31);
        if (!(lbm[t >> 5] & bit)) atomicOr(&lbm[t >> 5], bit);   // a stale 0 only costs the atomic
    }
    __syncthreads();
    for (int x = threadIdx.x; x < words; x += blockDim.x) {
        const uint32_t v = lbm[x];
        if (v && (v & ~__atomic_load_n(&bm[x], __ATOMIC_RELAXED))) atomicOr(&bm[x], v);
    }
}

__global__ __launch_bounds__(1024) void bitmap_count_kernel(const uint32_t *__restrict__ bm,
                                                            int words,
                                                            uint32_t *__restrict__ block_cnt)
{
    __shared__ uint32_t wsum[16];
    const int t = threadIdx.x;
    const int x = blockIdx.x * 1024 + t;
    uint32_t c = x < words ? __popc(bm[x]) : 0u;
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);
    if ((t & 63) == 0) wsum[t >> 6] = c;
    __syncthreads();
    if (t == 0) {
        uint32_t s = 0;
        for (int w = 0; w < 16; ++w) s += wsum[w];
        block_cnt[blockIdx.x] = s;
    }
}

__global__ __launch_bounds__(1024) void bitmap_write_kernel(const uint32_t *__restrict__ bm,
                                                            int words,
                                                            const uint32_t *__restrict__ block_off,
                                                            int32_t *__restrict__ unique)
{
    __shared__ uint32_t part[1024];
    const int t = threadIdx.x;
    const int x = blockIdx.x * 1024 + t;
    uint32_t w = x < words ? bm[x] : 0u;
    const uint32_t c = __popc(w);
    part[t] = c;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        uint32_t o = (t >= off) ? part[t - off] : 0u;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    uint32_t pos = block_off[blockIdx.x] + part[t] - c;
    while (w) {                                   // set bits, lowest first
        const int b = __ffs(w) - 1;
        unique[pos++] = (x << 5) + b;
        w &= w - 1;
    }
}

// ---------------------------------------------------------------- candidate lists

__global__ void pick_candidates_kernel(const int32_t *__restrict__ distinct,
                                       const uint32_t *__restrict__ n_distinct_p, int n_quantiles,
                                       int32_t *__restrict__ cand, SolveState *state, int cap)
{
    const int n = (int)*n_distinct_p;
    int C = (n_quantiles == 0 || n <= n_quantiles) ? n : n_quantiles;
    if (C > cap) C = cap;
    const bool all = (C == n);
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < C; j += gridDim.x * blockDim.x)
        cand[j] = all ? distinct[j] : distinct[((long long)j * (n - 1)) / (n_quantiles - 1)];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state->n_cand = C;
        state->n_distinct = n;
    }
}

__global__ void set_candidates_kernel(const uint32_t *__restrict__ n_unique_p, SolveState *state)
{
    state->n_cand = (int)*n_unique_p;
    state->n_distinct = (int)*n_unique_p;
}

// rank_of_orig[j] = index of tmax[j] in the ascending distinct list (binary search)
__global__ void rank_lookup_kernel(const int32_t *__restrict__ tmax, int n,
                                   const int32_t *__restrict__ unique,
                                   const uint32_t *__restrict__ n_unique_p,
                                   int32_t *__restrict__ rank_of_orig)
{
    const int nu = (int)*n_unique_p;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
        const int32_t x = tmax[j];
        int lo = 0, hi = nu;              // first index with unique[idx] >= x
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (unique[mid] < x) lo = mid + 1; else hi = mid;
        }
        rank_of_orig[j] = (lo < nu && unique[lo] == x) ? lo : -1;
    }
}

// ---------------------------------------------------------------- launchers

hipError_t launch_gather_table_values(hipStream_t st, const int32_t *table, int K, int S,
                                      int32_t inf_key, int32_t *out_keys)
{
    long long total = (long long)K * K * K * S;
    int grid = (int)((total + 255) / 256);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(gather_table_values_kernel, dim3(grid), dim3(256), 0, st, table, K, S,
                       inf_key, out_keys);
    return hipGetLastError();
}

// Sorts keys[0][0..n) (clobbering both key buffers), writes the ascending distinct values
// other than drop_key to out_unique and their count to *out_n_unique (device).
hipError_t launch_sort_dedup(hipStream_t st, PrepBuffers &pb, int n, int key_bits,
                             int32_t drop_key, int32_t *out_unique, uint32_t *out_n_unique)
{
    int cur = 0;
    for (int shift = 0; shift < key_bits; shift += 8) {
        hipLaunchKernelGGL(radix_hist_kernel, dim3(SORT_BLOCKS), dim3(WAVE), 0, st,
                           pb.keys[cur], n, shift, pb.hist);
        uint32_t *totals = pb.hist + RADIX * SORT_BLOCKS;
        hipLaunchKernelGGL(digit_scan_kernel, dim3(RADIX), dim3(SORT_BLOCKS), 0, st, pb.hist,
                           totals);
        hipLaunchKernelGGL(digit_base_kernel, dim3(1), dim3(RADIX), 0, st, totals);
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(SORT_BLOCKS), dim3(WAVE), 0, st,
                           pb.keys[cur], pb.keys[cur ^ 1], n, shift, pb.hist, totals);
        cur ^= 1;
    }
    const int nb = (n + DEDUP_TILE - 1) / DEDUP_TILE;
    hipLaunchKernelGGL(dedup_count_kernel, dim3(nb), dim3(1024), 0, st, pb.keys[cur], n, drop_key,
                       pb.block_cnt);
    hipLaunchKernelGGL(scan_u32_kernel, dim3(1), dim3(1024), 0, st, pb.block_cnt, nb,
                       out_n_unique);
    hipLaunchKernelGGL(dedup_write_kernel, dim3(nb), dim3(1024), 0, st, pb.keys[cur], n, drop_key,
                       pb.block_cnt, out_unique);
    return hipGetLastError();
}

// Ascending distinct finite values of the table's entries with last >= first layer, all known
// to be <= max_value < DISTINCT_BITMAP_MAX, to out_unique and their count to *out_n_unique.
// `work` holds the bitmap and the block counts: distinct_bitmap_words(max_value) uint32.
hipError_t launch_distinct_by_bitmap(hipStream_t st, const int32_t *table, int K, int S,
                                     int32_t max_value, uint32_t *work, int32_t *out_unique,
                                     uint32_t *out_n_unique)
{
    const int words = max_value / 32 + 1;
    const int nb = (words + 1023) / 1024;
    uint32_t *bm = work, *block_cnt = work + words;
    hipLaunchKernelGGL(bitmap_clear_kernel, dim3(std::min(nb, 256)), dim3(1024), 0, st, bm, words);
    const long long total = (long long)K * K * K * S;
    const int grid = (int)std::min<long long>((total + 8191) / 8192, 256);
    hipLaunchKernelGGL(bitmap_mark_kernel, dim3(grid), dim3(1024), (size_t)words * 4, st, table, K,
                       S, words, bm);
    hipLaunchKernelGGL(bitmap_count_kernel, dim3(nb), dim3(1024), 0, st, bm, words, block_cnt);
    hipLaunchKernelGGL(scan_u32_kernel, dim3(1), dim3(1024), 0, st, block_cnt, nb, out_n_unique);
    hipLaunchKernelGGL(bitmap_write_kernel, dim3(nb), dim3(1024), 0, st, bm, words, block_cnt,
                       out_unique);
    return hipGetLastError();
}

size_t distinct_bitmap_words(int32_t max_value)
{
    const size_t words = (size_t)max_value / 32 + 1;
    return words + (words + 1023) / 1024 + 1;
}

hipError_t launch_pick_candidates(hipStream_t st, const int32_t *distinct,
                                  const uint32_t *n_distinct, int n_quantiles, int32_t *cand,
                                  SolveState *state, int cap)
{
    int grid = (cap + 255) / 256;
    if (grid > 1024) grid = 1024;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(pick_candidates_kernel, dim3(grid), dim3(256), 0, st, distinct, n_distinct,
                       n_quantiles, cand, state, cap);
    return hipGetLastError();
}

hipError_t launch_set_candidates(hipStream_t st, const uint32_t *n_unique, SolveState *state)
{
    hipLaunchKernelGGL(set_candidates_kernel, dim3(1), dim3(1), 0, st, n_unique, state);
    return hipGetLastError();
}

hipError_t launch_rank_lookup(hipStream_t st, const int32_t *tmax, int n, const int32_t *unique,
                              const uint32_t *n_unique, int32_t *rank_of_orig)
{
    int grid = (n + 255) / 256;
    if (grid > 1024) grid = 1024;
    hipLaunchKernelGGL(rank_lookup_kernel, dim3(grid), dim3(256), 0, st, tmax, n, unique, n_unique,
                       rank_of_orig);
    return hipGetLastError();
}

}  // namespace alpa
