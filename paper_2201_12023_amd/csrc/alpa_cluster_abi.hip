// C ABI of the operator-clustering step: argument checks, device buffers, launch order.
#include "../../include/alpa_dp.h"
#include "internal.hpp"

#include <string>
#include <vector>

using namespace alpa;

extern "C" __attribute__((visibility("hidden"))) int alpa_dp_set_error_(int code, const char *msg);   // alpa_dp_abi.hip

namespace {

struct DevBuf {                       // frees on scope exit
    void *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 4); }
    template <class T> T *as() const { return (T *)p; }
};

int fail(int code, const std::string &msg) { return alpa_dp_set_error_(code, msg.c_str()); }

#define HIPCHK(expr)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(e_ == hipErrorOutOfMemory ? ALPA_DP_ENOMEM : ALPA_DP_EHIP,          \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                 \
    } while (0)

}  // namespace

static int cluster_layers_impl(const int32_t *flop, int K, const int32_t *edge_src,
                               const int32_t *edge_dst, const int64_t *edge_bytes, int num_edges,
                               int L, int delta_ppm, int64_t *out_comm, int64_t *out_sumsq,
                               int32_t *out_first_op, float *out_ms, int exact)
{
    if (!flop || !out_comm || !out_sumsq || !out_first_op)
        return fail(ALPA_DP_EINVAL, "null argument");
    if (K < 1 || K > ALPA_CLUSTER_MAX_OPS) return fail(ALPA_DP_EINVAL, "K out of range");
    if (L < 1 || L > ALPA_CLUSTER_MAX_OPS) return fail(ALPA_DP_EINVAL, "L out of range");
    if (num_edges < 0 || (num_edges > 0 && (!edge_src || !edge_dst || !edge_bytes)))
        return fail(ALPA_DP_EINVAL, "edge list is null or num_edges < 0");
    if (delta_ppm < 0 || delta_ppm > 1000000000) return fail(ALPA_DP_EINVAL, "delta_ppm out of range");
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        if (flop[k] < 0) return fail(ALPA_DP_EINVAL, "negative FLOP figure");
        total += flop[k];
    }
    if (total >= (1ll << 31)) return fail(ALPA_DP_EOVERFLOW, "total FLOP >= 2^31");
    if (total * (int64_t)L >= (1ll << 42)) return fail(ALPA_DP_EOVERFLOW, "total FLOP * L >= 2^42");
    int64_t all_bytes = 0;
    for (int e = 0; e < num_edges; ++e) {
        if (edge_src[e] < 0 || edge_dst[e] >= K || edge_src[e] >= edge_dst[e])
            return fail(ALPA_DP_EINVAL, "edge must go from an earlier to a later operator");
        if (edge_bytes[e] < 0) return fail(ALPA_DP_EINVAL, "negative edge size");
        if (edge_bytes[e] >= (1ll << 62) - all_bytes)
            return fail(ALPA_DP_EOVERFLOW, "sum of edge sizes >= 2^62");
        all_bytes += edge_bytes[e];
    }
    // FLOP(i..n) * L * 10^6 <= (10^6 + delta_ppm) * total, for integers, is FLOP(i..n) <= cap
    const int64_t cap = ((1000000ll + delta_ppm) * total) / ((int64_t)L * 1000000ll);

    hipStream_t st = nullptr;
    DevBuf d_flop, d_src, d_dst, d_nb, d_Ct, d_chunk, d_pf, d_GV, d_arg, d_out, d_first;
    const size_t E = (size_t)num_edges, Kp = (size_t)K + 1;
    HIPCHK(d_flop.alloc((size_t)K * 4));
    HIPCHK(d_src.alloc(E * 4));
    HIPCHK(d_dst.alloc(E * 4));
    HIPCHK(d_nb.alloc(E * 8));
    HIPCHK(d_Ct.alloc((size_t)K * K * 8));
    HIPCHK(d_chunk.alloc(cluster_chunk_rows(K) * K * 8));
    HIPCHK(d_pf.alloc(Kp * 8));
    HIPCHK(d_GV.alloc(4 * Kp * 8));
    HIPCHK(d_arg.alloc((size_t)L * Kp * 4));
    HIPCHK(d_out.alloc(2 * 8));
    HIPCHK(d_first.alloc(((size_t)L + 1) * 4));
    HIPCHK(hipMemcpyAsync(d_flop.p, flop, (size_t)K * 4, hipMemcpyHostToDevice, st));
    if (E) {
        HIPCHK(hipMemcpyAsync(d_src.p, edge_src, E * 4, hipMemcpyHostToDevice, st));
        HIPCHK(hipMemcpyAsync(d_dst.p, edge_dst, E * 4, hipMemcpyHostToDevice, st));
        HIPCHK(hipMemcpyAsync(d_nb.p, edge_bytes, E * 8, hipMemcpyHostToDevice, st));
    }
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    HIPCHK(hipEventCreate(&ev0));
    HIPCHK(hipEventCreate(&ev1));
    struct EvGuard { hipEvent_t a, b; ~EvGuard() { (void)hipEventDestroy(a); (void)hipEventDestroy(b); } }
        guard{ev0, ev1};
    HIPCHK(hipEventRecord(ev0, st));
    HIPCHK(launch_cluster(st, d_flop.as<int32_t>(), d_src.as<int32_t>(), d_dst.as<int32_t>(),
                          d_nb.as<int64_t>(), num_edges, K, L, cap, d_Ct.as<int64_t>(),
                          d_chunk.as<int64_t>(), d_pf.as<int64_t>(), d_GV.as<int64_t>(),
                          d_arg.as<int32_t>(), d_out.as<int64_t>(), d_first.as<int32_t>(), nullptr, 0,
                          exact));
    HIPCHK(hipEventRecord(ev1, st));
    int64_t res[2] = {0, 0};
    HIPCHK(hipMemcpyAsync(res, d_out.p, sizeof(res), hipMemcpyDeviceToHost, st));
    HIPCHK(hipMemcpyAsync(out_first_op, d_first.p, ((size_t)L + 1) * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    *out_comm = res[0];
    *out_sumsq = res[1];
    if (out_ms) HIPCHK(hipEventElapsedTime(out_ms, ev0, ev1));
    return ALPA_DP_OK;
}

extern "C" int alpa_cluster_layers(const int32_t *flop, int K, const int32_t *edge_src,
                                   const int32_t *edge_dst, const int64_t *edge_bytes,
                                   int num_edges, int L, int delta_ppm, int64_t *out_comm,
                                   int64_t *out_sumsq, int32_t *out_first_op, float *out_ms)
{
    return cluster_layers_impl(flop, K, edge_src, edge_dst, edge_bytes, num_edges, L, delta_ppm,
                               out_comm, out_sumsq, out_first_op, out_ms, 0);
}

extern "C" int alpa_cluster_layers_exact(const int32_t *flop, int K, const int32_t *edge_src,
                                         const int32_t *edge_dst, const int64_t *edge_bytes,
                                         int num_edges, int L, int delta_ppm, int64_t *out_comm,
                                         int64_t *out_sumsq, int32_t *out_first_op, float *out_ms)
{
    return cluster_layers_impl(flop, K, edge_src, edge_dst, edge_bytes, num_edges, L, delta_ppm,
                               out_comm, out_sumsq, out_first_op, out_ms, 1);
}

// ---------------------------------------------------------------- no allocation on the call

// Work memory of alpa_cluster_layers_static: what alpa_cluster_layers allocates per call, at
// the sizes of ALPA_CLUSTER_STATIC_MAX_OPS operators and layers, in int64 units:
// Ct [K*K], chunk [ceil(K/64)*K], pf [K+1], GV [4*(K+1)], ctl [8], arg [L*(K+1)] int32.
namespace {
constexpr size_t SMAX = ALPA_CLUSTER_STATIC_MAX_OPS;
constexpr size_t SCRATCH_I64 = SMAX * SMAX + ((SMAX + 63) / 64) * SMAX + (SMAX + 1) +
                               4 * (SMAX + 1) + 8 + (SMAX * (SMAX + 1) + 1) / 2;
}
// Every device the library runs on holds its own copy of this array until the process ends.  In
// host code the name is only a handle for hipGetSymbolAddress; kernels get the address below.
static __device__ __align__(256) int64_t scratch[SCRATCH_I64];

namespace {
constexpr int MAX_DEV = 64;
int64_t *g_scratch_of_device[MAX_DEV];      // device address of `scratch`, per device
bool g_scratch_known[MAX_DEV];
}

extern "C" int alpa_cluster_layers_static(const int32_t *d_flop, int K, const int32_t *d_edge_src,
                                          const int32_t *d_edge_dst, const int64_t *d_edge_bytes,
                                          int num_edges, int L, int delta_ppm, int64_t *d_out,
                                          int32_t *d_out_first_op, void *hip_stream)
{
    if (!d_flop || !d_out || !d_out_first_op) return fail(ALPA_DP_EINVAL, "null argument");
    if (K < 1 || L < 1) return fail(ALPA_DP_EINVAL, "K or L < 1");
    if (K > ALPA_CLUSTER_STATIC_MAX_OPS || L > ALPA_CLUSTER_STATIC_MAX_OPS)
        return fail(ALPA_DP_EINVAL, "K or L exceeds ALPA_CLUSTER_STATIC_MAX_OPS (the fixed work "
                                    "memory of this entry point); use alpa_cluster_layers");
    if (num_edges < 0 || (num_edges > 0 && (!d_edge_src || !d_edge_dst || !d_edge_bytes)))
        return fail(ALPA_DP_EINVAL, "edge list is null or num_edges < 0");
    if (delta_ppm < 0 || delta_ppm > 1000000000) return fail(ALPA_DP_EINVAL, "delta_ppm out of range");
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEV) return fail(ALPA_DP_EINVAL, "device index out of range");
    if (!g_scratch_known[dev]) {                   // set-up, once per device, that device current
        int64_t *ptr = nullptr;
        HIPCHK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(ALPA_DP_EHIP, "hipGetSymbolAddress gave a null address");
        g_scratch_of_device[dev] = ptr;
        g_scratch_known[dev] = true;
    }
    int64_t *base = g_scratch_of_device[dev];
    const size_t Ks = (size_t)K;
    int64_t *Ct = base;
    int64_t *chunk = Ct + Ks * Ks;
    int64_t *pf = chunk + cluster_chunk_rows(K) * Ks;
    int64_t *GV = pf + (Ks + 1);
    int64_t *ctl = GV + 4 * (Ks + 1);
    int32_t *arg = (int32_t *)(ctl + 8);
    // Everything the kernels read from the work memory they have written in this call (Ct is
    // cleared by a fill kernel, not a memset, so that the call can be recorded into a graph).
    HIPCHK(launch_cluster((hipStream_t)hip_stream, d_flop, d_edge_src, d_edge_dst, d_edge_bytes,
                          num_edges, K, L, /*cap=*/0, Ct, chunk, pf, GV, arg, d_out, d_out_first_op,
                          ctl, delta_ppm));
    return ALPA_DP_OK;
}
