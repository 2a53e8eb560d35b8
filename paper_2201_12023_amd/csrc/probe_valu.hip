// Measurement aid, not part of the method: a register-only loop of the recurrence's two vector
// instructions, and the entry point that times it.
#include "../../include/alpa_dp.h"
#include "internal.hpp"

#include <string>

// Register-only add + min chains (the two vector instructions of one cell-update, the add with
// a scalar operand as in the recurrence kernel) at full occupancy: what the int32 vector ALU
// can sustain, to set beside the nominal 256 CU x 64 lanes x clock figure.
namespace alpa {

struct Scalars16 { int32_t v[16]; };

__global__ __launch_bounds__(256) void valu_peak_kernel(int iters, Scalars16 sv,
                                                        int32_t *__restrict__ sink)
{
    int32_t a[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) a[u] = DEV_INF - (int)threadIdx.x - u;
    int32_t g = (int32_t)threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 8; ++rep) {
            // the sixteen sums (distinct scalar operands) before the sixteen minima, as the
            // recurrence kernel orders them: a minimum right behind its own sum holds the wave up
            int32_t sum[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) sum[u] = sv.v[u] + g;
            asm volatile("" : "+v"(sum[0]), "+v"(sum[1]), "+v"(sum[2]), "+v"(sum[3]), "+v"(sum[4]),
                              "+v"(sum[5]), "+v"(sum[6]), "+v"(sum[7]), "+v"(sum[8]), "+v"(sum[9]),
                              "+v"(sum[10]), "+v"(sum[11]), "+v"(sum[12]), "+v"(sum[13]),
                              "+v"(sum[14]), "+v"(sum[15]));
#pragma unroll
            for (int u = 0; u < 16; ++u) a[u] = min(a[u], sum[u]);
            // "everything may have changed": no repetition is folded away or fused with the next
            asm volatile("" : "+v"(g), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]),
                              "+v"(a[5]), "+v"(a[6]), "+v"(a[7]), "+v"(a[8]), "+v"(a[9]),
                              "+v"(a[10]), "+v"(a[11]), "+v"(a[12]), "+v"(a[13]), "+v"(a[14]),
                              "+v"(a[15]));
        }
        g = a[it & 15] ^ g;                       // keeps the chain from being folded
        asm volatile("" : "+v"(g));
    }
    int32_t r = g;
#pragma unroll
    for (int u = 0; u < 16; ++u) r = min(r, a[u]);
    if (r == 0x12345678) sink[0] = r;             // never true in practice; keeps the work alive
}

// 256 add/min instructions per iteration and thread are counted (the two chain-breaking ones not)
hipError_t launch_valu_peak(hipStream_t st, int grid, int iters, int32_t *sink)
{
    Scalars16 sv;
    for (int u = 0; u < 16; ++u) sv.v[u] = 3 + 2 * u;
    hipLaunchKernelGGL(valu_peak_kernel, dim3(grid), dim3(256), 0, st, iters, sv, sink);
    return hipGetLastError();
}

}  // namespace alpa

extern "C" __attribute__((visibility("hidden"))) int alpa_dp_set_error_(int code, const char *msg);   // alpa_dp_abi.hip

extern "C" int alpa_dp_measure_valu_peak(double *out_lane_ops_per_s)
{
    using namespace alpa;
    auto fail = [](int code, const std::string &msg) { return alpa_dp_set_error_(code, msg.c_str()); };
#define PROBE_CHK(expr)                                                                     \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            if (sink) (void)hipFree(sink);                                                  \
            if (ev0) (void)hipEventDestroy(ev0);                                            \
            if (ev1) (void)hipEventDestroy(ev1);                                            \
            return fail(e_ == hipErrorOutOfMemory ? ALPA_DP_ENOMEM : ALPA_DP_EHIP,          \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                 \
        }                                                                                   \
    } while (0)
    int32_t *sink = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (!out_lane_ops_per_s) return fail(ALPA_DP_EINVAL, "null argument");
    hipDeviceProp_t prop;
    int dev = 0;
    PROBE_CHK(hipGetDevice(&dev));
    PROBE_CHK(hipGetDeviceProperties(&prop, dev));
    PROBE_CHK(hipMalloc(&sink, 64));
    PROBE_CHK(hipEventCreate(&ev0));
    PROBE_CHK(hipEventCreate(&ev1));
    const int grid = prop.multiProcessorCount * 8, iters = 4000;       // 8 waves per SIMD
    PROBE_CHK(launch_valu_peak(nullptr, grid, 100, sink));             // warm-up
    PROBE_CHK(hipEventRecord(ev0, nullptr));
    PROBE_CHK(launch_valu_peak(nullptr, grid, iters, sink));
    PROBE_CHK(hipEventRecord(ev1, nullptr));
    PROBE_CHK(hipEventSynchronize(ev1));
    float ms = 0;
    PROBE_CHK(hipEventElapsedTime(&ms, ev0, ev1));
    (void)hipFree(sink);
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    *out_lane_ops_per_s = (double)grid * 256.0 * 256.0 * iters / (ms * 1e-3);
    return ALPA_DP_OK;
#undef PROBE_CHK
}
