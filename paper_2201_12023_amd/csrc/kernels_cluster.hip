// Operator clustering on the device (Sec. 5.2, performance optimisation #2, Eq. 6):
//   G(n, r) = min over 1 <= i <= n with FLOP(o_i..o_n) <= cap of max{G(i-1, r-1), C(i, n)},
// C(i, n) = bytes that o_i..o_n receive from o_1..o_{i-1}; ties go to the smaller sum of squared
// per-layer FLOP (carried as V(n, r)), then to the smaller i.
//
// Kernels: the edge list is added into a dense consumer-major matrix; an exclusive prefix along
// producers and a running sum down consumers turn it, in place, into Ct[n][i] = C(i, n) with
// the candidates i of one n contiguous; one launch per r then evaluates every n in parallel,
// one wave per n, lanes over i, with a lexicographic wave minimum; one thread walks the stored
// arg-minima back.  FLOP figures are non-negative, so the feasible i of an n form a suffix
// [i_min(n), n] found by bisection on the FLOP prefix sums: the work is K * (layer length) per r,
// not K^2.  Memory-bound on the reads of Ct.
#include "internal.hpp"

namespace alpa {

constexpr int CL_TILE = 64;            // rows per chunk of the column scan

// pf[x] = FLOP of operators 0..x-1 (int64), one block
__global__ __launch_bounds__(1024) void flop_prefix_kernel(const int32_t *__restrict__ flop, int K,
                                                           int64_t *__restrict__ pf)
{
    __shared__ int64_t part[1024];
    const int t = threadIdx.x;
    const int per = (K + 1023) / 1024;
    const int lo = min(K, t * per), hi = min(K, lo + per);
    int64_t s = 0;
    for (int x = lo; x < hi; ++x) s += flop[x];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const int64_t o = (t >= off) ? part[t - off] : 0;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    int64_t run = part[t] - s;
    if (t == 0) pf[0] = 0;
    for (int x = lo; x < hi; ++x) {
        run += flop[x];
        pf[x + 1] = run;
    }
}

__global__ void zero_i64_kernel(int64_t *p, long long n)
{
    for (long long x = blockIdx.x * (long long)blockDim.x + threadIdx.x; x < n;
         x += (long long)gridDim.x * blockDim.x)
        p[x] = 0;
}

// Wt[v][u] += bytes(u -> v)
__global__ void edges_to_matrix_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ dst,
                                       const int64_t *__restrict__ nbytes, int E, int K,
                                       int64_t *__restrict__ Wt)
{
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < E; e += gridDim.x * blockDim.x) {
        const int u = src[e], v = dst[e];
        // callers with host arrays have checked this already; with device arrays the check
        // kernel reports such an edge, and here it must not be written
        if (u < 0 || v >= K || u >= v) continue;
        atomicAdd((unsigned long long *)&Wt[(size_t)v * K + u], (unsigned long long)nbytes[e]);
    }
}

// Argument checks for device-resident inputs (what alpa_cluster_layers does on the host):
// ctl[0] = 0, ALPA_DP_EINVAL (-1: negative figure, bad edge) or ALPA_DP_EOVERFLOW (-2: total FLOP
// >= 2^31, total * L >= 2^42, edge sizes adding up to >= 2^62); ctl[1] = the FLOP bound per
// layer, floor((10^6 + delta_ppm) * total / (L * 10^6)).  One block.
__global__ __launch_bounds__(1024) void cluster_check_kernel(
    const int32_t *__restrict__ flop, int K, const int32_t *__restrict__ src,
    const int32_t *__restrict__ dst, const int64_t *__restrict__ nbytes, int E, int L,
    int delta_ppm, int64_t *__restrict__ ctl)
{
    __shared__ unsigned long long sh_flop, sh_bytes;
    __shared__ int sh_bad, sh_over;
    const int t = threadIdx.x;
    if (t == 0) { sh_flop = 0; sh_bytes = 0; sh_bad = 0; sh_over = 0; }
    __syncthreads();
    constexpr unsigned long long LIM = 1ull << 62;
    unsigned long long f = 0, b = 0;
    int bad = 0, over = 0;
    for (int k = t; k < K; k += 1024) {
        const int32_t v = flop[k];
        if (v < 0) bad = 1; else f += (unsigned long long)v;        // < 2^31 * 4 per thread
    }
    for (int e = t; e < E; e += 1024) {
        const int u = src[e], v = dst[e];
        const int64_t n = nbytes[e];
        if (u < 0 || v >= K || u >= v || n < 0) { bad = 1; continue; }
        if ((unsigned long long)n >= LIM) over = 1;
        b = min(LIM, b + min(LIM, (unsigned long long)n));         // saturating: stays <= 2^62
    }
    atomicAdd(&sh_flop, f);
    if (bad) atomicOr(&sh_bad, 1);
    if (over) atomicOr(&sh_over, 1);
    __syncthreads();
    // the byte total, saturating, one thread after the other (1024 partial sums <= 2^62 each
    // would wrap an unsigned 64-bit add)
    for (int turn = 0; turn < 1024; turn += WAVE) {
        if (t >= turn && t < turn + WAVE) {
            unsigned long long x = b;
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned long long o =
                    (unsigned long long)i64_from(__shfl_xor(lo32((int64_t)x), off, 64),
                                                 __shfl_xor(hi32((int64_t)x), off, 64));
                x = min(LIM, x + o);
            }
            if ((t & (WAVE - 1)) == 0) sh_bytes = min(LIM, sh_bytes + x);
        }
        __syncthreads();
    }
    if (t == 0) {
        const unsigned long long total = sh_flop;
        int64_t status = 0;
        if (sh_bad) status = -1;
        else if (total >= (1ull << 31) || total * (unsigned long long)L >= (1ull << 42) ||
                 sh_over || sh_bytes >= LIM) status = -2;
        ctl[0] = status;
        ctl[1] = status ? 0
                        : (int64_t)(((1000000ull + (unsigned long long)delta_ppm) * total) /
                                    ((unsigned long long)L * 1000000ull));
    }
}

// row v: A[v][i] = sum over u < i of Wt[v][u], i = 0..K-1, in place (one block per row)
__global__ __launch_bounds__(256) void row_prefix_kernel(int64_t *__restrict__ Wt, int K)
{
    __shared__ int64_t part[256];
    const int t = threadIdx.x;
    int64_t *row = Wt + (size_t)blockIdx.x * K;
    const int per = (K + 255) / 256;
    const int lo = min(K, t * per), hi = min(K, lo + per);
    int64_t s = 0;
    for (int x = lo; x < hi; ++x) s += row[x];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int64_t o = (t >= off) ? part[t - off] : 0;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    int64_t run = part[t] - s;
    for (int x = lo; x < hi; ++x) {
        const int64_t w = row[x];
        row[x] = run;
        run += w;
    }
}

// Column i: Ct[n][i] = sum over v = i..n of A[v][i] for n >= i (entries with n < i are not
// used).  Three passes over chunks of CL_TILE rows: chunk sums, their prefix, the running sum.
__global__ __launch_bounds__(64) void col_chunk_sum_kernel(const int64_t *__restrict__ A, int K,
                                                           int64_t *__restrict__ chunk)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int r0 = blockIdx.y * CL_TILE;
    if (i >= K) return;
    int64_t s = 0;
    const int r1 = min(K, r0 + CL_TILE);
    for (int v = max(r0, i); v < r1; ++v) s += A[(size_t)v * K + i];
    chunk[(size_t)blockIdx.y * K + i] = s;
}

__global__ void col_chunk_prefix_kernel(int64_t *__restrict__ chunk, int K, int n_chunks)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K) return;
    int64_t run = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t s = chunk[(size_t)c * K + i];
        chunk[(size_t)c * K + i] = run;
        run += s;
    }
}

__global__ __launch_bounds__(64) void col_running_sum_kernel(int64_t *__restrict__ A, int K,
                                                             const int64_t *__restrict__ chunk)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    const int r0 = blockIdx.y * CL_TILE;
    if (i >= K) return;
    int64_t run = chunk[(size_t)blockIdx.y * K + i];
    const int r1 = min(K, r0 + CL_TILE);
    for (int v = max(r0, i); v < r1; ++v) {
        run += A[(size_t)v * K + i];
        A[(size_t)v * K + i] = run;
    }
}

// G(., 0): only the empty prefix is finite
__global__ void cluster_init_kernel(int64_t *__restrict__ G, int64_t *__restrict__ V, int K)
{
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x <= K; x += gridDim.x * blockDim.x) {
        G[x] = (x == 0) ? 0 : INF_I64;
        V[x] = 0;
    }
}

struct Lex {                    // (G, V, i): smaller is better, component by component
    int64_t g, v;
    int i;
};
__device__ __forceinline__ bool lex_less(const Lex &a, const Lex &b)
{
    return a.g < b.g || (a.g == b.g && (a.v < b.v || (a.v == b.v && a.i < b.i)));
}
__device__ __forceinline__ Lex lex_shfl_xor(const Lex &a, int m)
{
    Lex o;
    o.g = i64_from(__shfl_xor(lo32(a.g), m, 64), __shfl_xor(hi32(a.g), m, 64));
    o.v = i64_from(__shfl_xor(lo32(a.v), m, 64), __shfl_xor(hi32(a.v), m, 64));
    o.i = __shfl_xor(a.i, m, 64);
    return o;
}

// One layer count r: Gn[n], Vn[n], arg[n] for n = 1..K from Gp, Vp (r - 1).  One wave per n.
__global__ __launch_bounds__(256) void cluster_layer_kernel(
    const int64_t *__restrict__ Ct, const int64_t *__restrict__ pf, int K, int64_t cap,
    const int64_t *__restrict__ ctl, const int64_t *__restrict__ Gp,
    const int64_t *__restrict__ Vp, int64_t *__restrict__ Gn, int64_t *__restrict__ Vn,
    int32_t *__restrict__ arg)
{
    if (ctl) cap = ctl[1];                          // bound computed on the device (cluster_check_kernel)
    const int lane = threadIdx.x & (WAVE - 1);
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6) + 1;          // prefix length, 1-based
    if (n > K) return;                                              // whole wave
    // smallest i (1-based) with pf[n] - pf[i-1] <= cap: bisection on the non-decreasing pf
    const int64_t need = pf[n] - cap;                               // pf[i-1] >= need
    int lo = 0, hi = n;                                             // answer index x = i-1 in [0, n]
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (pf[mid] >= need) hi = mid; else lo = mid + 1;
    }
    const int i_min = lo + 1;                                       // may be n + 1: nothing fits
    Lex best{INF_I64, 0, 0};
    const int64_t *row = Ct + (size_t)(n - 1) * K;                  // Ct[n-1][i-1] = C(i, n)
    for (int i = i_min + lane; i <= n; i += WAVE) {
        const int64_t gp = Gp[i - 1];
        if (gp == INF_I64) continue;
        const int64_t c = row[i - 1];
        const int64_t f = pf[n] - pf[i - 1];
        const Lex cur{gp > c ? gp : c, Vp[i - 1] + f * f, i};
        if (lex_less(cur, best)) best = cur;
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) {
        const Lex o = lex_shfl_xor(best, m);
        if (lex_less(o, best)) best = o;
    }
    if (best.g == INF_I64) { best.v = 0; best.i = 0; }
    Gn[n] = best.g;                                                 // all lanes, same value
    Vn[n] = best.v;
    arg[n] = best.i;
    if (lane == 0 && n == 1) { Gn[0] = INF_I64; Vn[0] = 0; arg[0] = 0; }   // G(0, r > 0)
}

// Second run of the exact mode (the variance tie-break over whole clusterings): with
// G* = G(K, L) of the first run in *gstar_p,
//   W(n, r) = min over the feasible i with C(i, n) <= G* of W(i-1, r-1) + FLOP(o_i..o_n)^2,
// lowest i on ties.  Same mapping as cluster_layer_kernel.
__global__ __launch_bounds__(256) void cluster_layer_exact_kernel(
    const int64_t *__restrict__ Ct, const int64_t *__restrict__ pf, int K, int64_t cap,
    const int64_t *__restrict__ gstar_p, const int64_t *__restrict__ Wp,
    int64_t *__restrict__ Wn, int32_t *__restrict__ arg)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6) + 1;
    if (n > K) return;                                              // whole wave
    const int64_t gstar = *gstar_p;
    const int64_t need = pf[n] - cap;
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (pf[mid] >= need) hi = mid; else lo = mid + 1;
    }
    const int i_min = lo + 1;
    Lex best{INF_I64, 0, 0};                                        // (W, unused, i)
    const int64_t *row = Ct + (size_t)(n - 1) * K;
    if (gstar != INF_I64) {
        for (int i = i_min + lane; i <= n; i += WAVE) {
            const int64_t wp = Wp[i - 1];
            if (wp == INF_I64 || row[i - 1] > gstar) continue;
            const int64_t f = pf[n] - pf[i - 1];
            const Lex cur{wp + f * f, 0, i};
            if (lex_less(cur, best)) best = cur;
        }
    }
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) {
        const Lex o = lex_shfl_xor(best, m);
        if (lex_less(o, best)) best = o;
    }
    if (best.g == INF_I64) best.i = 0;
    Wn[n] = best.g;                                                 // all lanes, same value
    arg[n] = best.i;
    if (lane == 0 && n == 1) { Wn[0] = INF_I64; arg[0] = 0; }       // W(0, r > 0)
}

// keep[0] = G(K, L) of the first run; W(., 0) for the second: only the empty prefix is finite
__global__ void cluster_begin_exact_kernel(const int64_t *__restrict__ G, int K,
                                           int64_t *__restrict__ keep, int64_t *__restrict__ W0)
{
    const int64_t g = G[K];                                         // read before W0 may alias it
    __syncthreads();
    for (int x = threadIdx.x; x <= K; x += blockDim.x) W0[x] = (x == 0) ? 0 : INF_I64;
    if (threadIdx.x == 0) keep[0] = g;
}

// out[0] = G(K, L), out[1] = V(K, L); first_op[0..L] by walking arg back (one thread).  With
// ctl (device-resident inputs) also out[2] = ctl[0], the status of the argument checks, and
// "no clustering" is reported if that is not 0.
__global__ void cluster_walk_kernel(const int64_t *__restrict__ G, const int64_t *__restrict__ V,
                                    const int32_t *__restrict__ arg, int K, int L,
                                    const int64_t *__restrict__ ctl, int64_t *__restrict__ out,
                                    int32_t *__restrict__ first_op,
                                    const int64_t *__restrict__ gstar_p)
{
    // gstar_p (exact mode): the first component is *gstar_p and V is the second run's W row
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    if (ctl) out[2] = ctl[0];
    const int64_t g = (ctl && ctl[0] != 0) ? INF_I64 : (gstar_p ? *gstar_p : G[K]);
    out[0] = g;
    out[1] = g == INF_I64 ? 0 : V[K];
    if (g == INF_I64) {
        for (int r = 0; r <= L; ++r) first_op[r] = -1;
        return;
    }
    int n = K;
    first_op[L] = K;
    for (int r = L; r >= 1; --r) {
        const int i = arg[(size_t)(r - 1) * (K + 1) + n];
        first_op[r - 1] = i - 1;
        n = i - 1;
    }
}

hipError_t launch_cluster(hipStream_t st, const int32_t *flop, const int32_t *src,
                          const int32_t *dst, const int64_t *nbytes, int E, int K, int L,
                          int64_t cap, int64_t *Ct, int64_t *chunk, int64_t *pf, int64_t *GV,
                          int32_t *arg, int64_t *out, int32_t *first_op, int64_t *ctl,
                          int delta_ppm, int exact)
{
    if (ctl)
        hipLaunchKernelGGL(cluster_check_kernel, dim3(1), dim3(1024), 0, st, flop, K, src, dst,
                           nbytes, E, L, delta_ppm, ctl);
    hipLaunchKernelGGL(flop_prefix_kernel, dim3(1), dim3(1024), 0, st, flop, K, pf);
    const long long kk = (long long)K * K;
    hipLaunchKernelGGL(zero_i64_kernel, dim3((unsigned)std::min<long long>((kk + 255) / 256, 4096)),
                       dim3(256), 0, st, Ct, kk);
    if (E > 0)
        hipLaunchKernelGGL(edges_to_matrix_kernel, dim3((E + 255) / 256), dim3(256), 0, st, src, dst,
                           nbytes, E, K, Ct);
    hipLaunchKernelGGL(row_prefix_kernel, dim3(K), dim3(256), 0, st, Ct, K);
    const int n_chunks = (K + CL_TILE - 1) / CL_TILE;
    const dim3 cgrid((K + 63) / 64, n_chunks);
    hipLaunchKernelGGL(col_chunk_sum_kernel, cgrid, dim3(64), 0, st, Ct, K, chunk);
    hipLaunchKernelGGL(col_chunk_prefix_kernel, dim3((K + 255) / 256), dim3(256), 0, st, chunk, K,
                       n_chunks);
    hipLaunchKernelGGL(col_running_sum_kernel, cgrid, dim3(64), 0, st, Ct, K, chunk);
    // GV: G and V rows of two consecutive layer counts, [2][2][K + 1]
    int64_t *G[2] = {GV, GV + 2 * (size_t)(K + 1)};
    int64_t *V[2] = {GV + (K + 1), GV + 3 * (size_t)(K + 1)};
    hipLaunchKernelGGL(cluster_init_kernel, dim3((K + 256) / 256), dim3(256), 0, st, G[0], V[0], K);
    for (int r = 1; r <= L; ++r) {
        const int p = (r - 1) & 1, c = r & 1;
        hipLaunchKernelGGL(cluster_layer_kernel, dim3((K + 3) / 4), dim3(256), 0, st, Ct, pf, K, cap,
                           (const int64_t *)ctl, G[p], V[p], G[c], V[c],
                           arg + (size_t)(r - 1) * (K + 1));
    }
    if (exact) {
        // second run over the V rows (the first run's V values are not needed any more);
        // G* is parked in the G row that the first run wrote last but one
        int64_t *keep = G[(L & 1) ^ 1];
        hipLaunchKernelGGL(cluster_begin_exact_kernel, dim3(1), dim3(256), 0, st, G[L & 1], K, keep,
                           V[0]);
        for (int r = 1; r <= L; ++r) {
            const int p = (r - 1) & 1, c = r & 1;
            hipLaunchKernelGGL(cluster_layer_exact_kernel, dim3((K + 3) / 4), dim3(256), 0, st, Ct,
                               pf, K, cap, (const int64_t *)keep, V[p], V[c],
                               arg + (size_t)(r - 1) * (K + 1));
        }
        hipLaunchKernelGGL(cluster_walk_kernel, dim3(1), dim3(WAVE), 0, st, V[L & 1], V[L & 1], arg,
                           K, L, (const int64_t *)ctl, out, first_op, (const int64_t *)keep);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(cluster_walk_kernel, dim3(1), dim3(WAVE), 0, st, G[L & 1], V[L & 1], arg, K, L,
                       (const int64_t *)ctl, out, first_op, (const int64_t *)nullptr);
    return hipGetLastError();
}

size_t cluster_chunk_rows(int K) { return (size_t)((K + CL_TILE - 1) / CL_TILE); }

}  // namespace alpa
