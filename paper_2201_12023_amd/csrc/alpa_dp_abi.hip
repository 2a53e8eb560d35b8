// C ABI of libalpa_dp: argument checks, device buffers, and the order in which the
// kernels of one solve are queued.  All arithmetic of the method is in the kernels.
#include "../../include/alpa_dp.h"
#include "internal.hpp"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace alpa;

static_assert(sizeof(alpa_plan_t) == 2072, "plan layout differs from the kernels' PlanDev");

static thread_local std::string g_err;

static int fail(int code, const std::string &msg)
{
    g_err = msg;
    return code;
}

// for the library's other translation units: same thread-local message
extern "C" __attribute__((visibility("hidden"))) int alpa_dp_set_error_(int code, const char *msg)
{
    return fail(code, msg);
}

#define HIPCHK(expr)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(e_ == hipErrorOutOfMemory ? ALPA_DP_ENOMEM : ALPA_DP_EHIP,          \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                 \
    } while (0)

struct alpa_dp {
    Problem p{};
    int device = 0;
    hipStream_t stream = nullptr;
    int32_t max_finite = -1;        // largest finite table entry with last >= first layer
    int key_bits_table = 1;
    int n_table_keys = 0;           // K * K(K+1)/2 * S
    int n_distinct = 0;             // distinct finite table values
    int n_cu = 0;
    bool fast_ok = false;
    int KP = 0;
    int fast_grid_max[3] = {0, 0, 0}, generic_grid_max = 0;   // [nc] for nc = 1, 2

    int32_t *d_table = nullptr, *d_sizes = nullptr, *d_recs = nullptr, *d_gmin = nullptr;
    PrepBuffers pb{};
    int32_t *d_distinct = nullptr;
    uint32_t *d_ncount = nullptr;   // [2]: distinct table values, distinct caller candidates
    int32_t *d_cand = nullptr, *d_rank = nullptr, *d_tmax_stage = nullptr;
    int32_t *d_Fmin = nullptr, *d_Sbest = nullptr;
    int64_t *d_T = nullptr, *d_outT_stage = nullptr, *d_chunkmin = nullptr;
    int cand_cap = 0;               // capacity of the per-candidate arrays
    SolveState *d_state = nullptr;
    int32_t *d_scratch = nullptr, *d_Fall = nullptr, *d_tmpFS = nullptr;
    alpa_plan_t *d_plan_tmp = nullptr, *d_best_plan = nullptr;
    // sweep over B (allocated on first use, for up to sw_cap values)
    int sw_cap = 0;
    int32_t *d_sw_B = nullptr, *d_sw_c = nullptr, *d_sw_s = nullptr, *d_sw_FS = nullptr;
    int32_t *d_sw_n = nullptr;      // [2]: number of B values, ticket of the plan-recovery run
    SolveState *d_sw_state = nullptr;
    int32_t *d_sw_Fall = nullptr;
    alpa_plan_t *d_sw_plans = nullptr;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    bool any_solve = false, timed = false;
    bool have_best = false;         // d_best_plan holds the best of a solve made with the current
                                    // table and B (sweeps do not touch it)
    // tuning (alpa_dp_set_tuning); 0 = the library's own choice
    int tune_nc = 0, tune_sort = 0, tune_wg_per_cu = 0, tune_grid = 0, tune_no_groups = 0;
    int fast_per_cu[3] = {0, 0, 0};  // resident workgroups per compute unit, [nc]
};

static void free_candidate_arrays(alpa_dp *h)
{
    (void)hipFree(h->pb.keys[0]); (void)hipFree(h->pb.keys[1]); (void)hipFree(h->pb.block_cnt);
    (void)hipFree(h->d_cand); (void)hipFree(h->d_rank); (void)hipFree(h->d_tmax_stage);
    (void)hipFree(h->d_Fmin); (void)hipFree(h->d_Sbest); (void)hipFree(h->d_T); (void)hipFree(h->d_outT_stage);
    (void)hipFree(h->d_chunkmin); (void)hipFree(h->d_distinct);
    h->pb.keys[0] = h->pb.keys[1] = nullptr; h->pb.block_cnt = nullptr;
    h->d_cand = h->d_rank = h->d_tmax_stage = h->d_Fmin = h->d_Sbest = h->d_distinct = nullptr;
    h->d_T = h->d_outT_stage = h->d_chunkmin = nullptr;
    h->cand_cap = 0;
    h->pb.cap = 0;
}

// Per-candidate arrays for up to `cap` keys / candidates.  All or nothing: after a failure
// every pointer is null and both capacities are 0, so the next solve tries again (and fails
// with ENOMEM again rather than launching on short buffers).
static int alloc_candidate_arrays(alpa_dp *h, int cap)
{
    free_candidate_arrays(h);
    const size_t c = (size_t)cap;
    auto body = [&]() -> int {
        HIPCHK(hipMalloc(&h->pb.keys[0], c * 4));
        HIPCHK(hipMalloc(&h->pb.keys[1], c * 4));
        HIPCHK(hipMalloc(&h->pb.block_cnt, (c / 4096 + 2) * 4));
        HIPCHK(hipMalloc(&h->d_distinct, c * 4));
        HIPCHK(hipMalloc(&h->d_cand, c * 4));
        HIPCHK(hipMalloc(&h->d_rank, c * 4));
        HIPCHK(hipMalloc(&h->d_tmax_stage, c * 4));
        HIPCHK(hipMalloc(&h->d_Fmin, (c + 1) * 4));      // + one spare slot (see FastArgs)
        HIPCHK(hipMalloc(&h->d_Sbest, (c + 1) * 4));
        HIPCHK(hipMalloc(&h->d_T, c * 8));
        HIPCHK(hipMalloc(&h->d_outT_stage, c * 8));
        HIPCHK(hipMalloc(&h->d_chunkmin, (c / PRUNE_CHUNK + 2) * 8));
        return ALPA_DP_OK;
    };
    const int rc = body();
    if (rc != ALPA_DP_OK) {
        free_candidate_arrays(h);
        return rc;
    }
    h->pb.cap = cap;
    h->cand_cap = cap;
    return ALPA_DP_OK;
}

// Capacity every solve needs: the table's keys for the sort of its values, and the caller's
// list if that is longer.
static int ensure_candidate_arrays(alpa_dp *h, int n_list)
{
    const int need = std::max(std::max(h->n_table_keys, 1024), n_list);
    if (h->cand_cap >= need) return ALPA_DP_OK;
    HIPCHK(hipStreamSynchronize(h->stream));
    return alloc_candidate_arrays(h, need);
}

static void free_sweep_arrays(alpa_dp *h)
{
    (void)hipFree(h->d_sw_B); (void)hipFree(h->d_sw_c); (void)hipFree(h->d_sw_s);
    (void)hipFree(h->d_sw_FS); (void)hipFree(h->d_sw_n); (void)hipFree(h->d_sw_state);
    (void)hipFree(h->d_sw_Fall); (void)hipFree(h->d_sw_plans);
    h->d_sw_B = h->d_sw_c = h->d_sw_s = h->d_sw_FS = h->d_sw_n = h->d_sw_Fall = nullptr;
    h->d_sw_state = nullptr;
    h->d_sw_plans = nullptr;
    h->sw_cap = 0;
}

static int alloc_sweep_arrays(alpa_dp *h, int n_B)
{
    free_sweep_arrays(h);
    const size_t n = (size_t)n_B;
    HIPCHK(hipMalloc(&h->d_sw_B, n * 4));
    HIPCHK(hipMalloc(&h->d_sw_c, n * 4));
    HIPCHK(hipMalloc(&h->d_sw_s, n * 4));
    HIPCHK(hipMalloc(&h->d_sw_FS, 2 * (n + 1) * 4));
    HIPCHK(hipMalloc(&h->d_sw_n, 2 * 4));
    HIPCHK(hipMalloc(&h->d_sw_state, n * sizeof(SolveState)));
    HIPCHK(hipMalloc(&h->d_sw_plans, n * sizeof(alpa_plan_t)));
    if (h->fast_ok && h->p.D <= 64) {   // one slab of layers per B value; the general kernel (also
                                        // used above 64 devices) reuses d_Fall
        const size_t slab = (size_t)(h->p.Smax + 1) * (size_t)(h->p.K + 2) * (h->p.D + 1);
        HIPCHK(hipMalloc(&h->d_sw_Fall, n * slab * 4));
    }
    h->sw_cap = n_B;
    return ALPA_DP_OK;
}

static int bits_for(uint32_t v)
{
    int b = 1;
    while (b < 32 && (v >> b)) ++b;
    return b;
}

// distinct finite table values -> d_distinct, count -> d_ncount[0]
static int queue_table_candidates(alpa_dp *h)
{
    // small values: one bit per value instead of a sort (the second key buffer is the work area)
    if (h->max_finite >= 0 && h->max_finite < DISTINCT_BITMAP_MAX && !h->tune_sort &&
        distinct_bitmap_words(h->max_finite) <= (size_t)h->pb.cap) {
        HIPCHK(launch_distinct_by_bitmap(h->stream, h->d_table, h->p.K, h->p.S, h->max_finite,
                                         (uint32_t *)h->pb.keys[1], h->d_distinct,
                                         h->d_ncount + 0));
        return ALPA_DP_OK;
    }
    const int32_t inf_key = h->max_finite + 1;
    HIPCHK(launch_gather_table_values(h->stream, h->d_table, h->p.K, h->p.S, inf_key,
                                      h->pb.keys[0]));
    HIPCHK(launch_sort_dedup(h->stream, h->pb, h->n_table_keys, h->key_bits_table, inf_key,
                             h->d_distinct, h->d_ncount + 0));
    return ALPA_DP_OK;
}

extern "C" const char *alpa_dp_last_error(void) { return g_err.c_str(); }

extern "C" void alpa_dp_destroy(alpa_dp_t *h)
{
    if (!h) return;
    int prev = 0;
    (void)hipGetDevice(&prev);
    (void)hipSetDevice(h->device);
    (void)hipStreamSynchronize(h->stream);
    free_candidate_arrays(h);
    free_sweep_arrays(h);
    (void)hipFree(h->d_table); (void)hipFree(h->d_sizes); (void)hipFree(h->d_recs); (void)hipFree(h->d_gmin);
    (void)hipFree(h->pb.hist); (void)hipFree(h->d_ncount); (void)hipFree(h->d_state); (void)hipFree(h->d_scratch);
    (void)hipFree(h->d_Fall); (void)hipFree(h->d_tmpFS); (void)hipFree(h->d_plan_tmp); (void)hipFree(h->d_best_plan);
    for (auto &e : h->ev) if (e) (void)hipEventDestroy(e);
    (void)hipSetDevice(prev);
    delete h;
}

// Argument checks common to both ways of creating a handle; fills sizes[q] = n_q * m_q.
static int check_problem(int K, int N, int M, int B, const alpa_shape_t *shapes, int num_shapes,
                         std::vector<int32_t> &sizes)
{
    if (!shapes) return fail(ALPA_DP_EINVAL, "shapes is null");
    if (K < 1 || K > ALPA_DP_MAX_K) return fail(ALPA_DP_EINVAL, "K out of range");
    if (N < 1 || M < 1 || (long long)N * M > ALPA_DP_MAX_DEVICES)
        return fail(ALPA_DP_EINVAL, "N x M out of range");
    if ((M & (M - 1)) != 0) return fail(ALPA_DP_EINVAL, "M must be a power of two");
    if (B < 1) return fail(ALPA_DP_EINVAL, "B must be >= 1");
    if (num_shapes < 1 || num_shapes > ALPA_DP_MAX_SHAPES)
        return fail(ALPA_DP_EINVAL, "num_shapes out of range");
    sizes.resize(num_shapes);
    for (int q = 0; q < num_shapes; ++q) {
        const int n = shapes[q].n, m = shapes[q].m;
        const bool one_d = n == 1 && m >= 1 && m <= M && (m & (m - 1)) == 0;
        const bool two_d = m == M && n >= 2 && n <= N;
        if (!one_d && !two_d) return fail(ALPA_DP_EINVAL, "shape outside the submesh family");
        sizes[q] = n * m;
    }
    return ALPA_DP_OK;
}

// Device side of handle creation.  `fill_table` puts the table into h->d_table (already
// allocated) and sets h->max_finite; everything else follows from those two.
template <class FillTable>
static int create_on_device(alpa_dp *h, const std::vector<int32_t> &sizes, FillTable fill_table)
{
    const int K = h->p.K, S = h->p.S, D = h->p.D;
    HIPCHK(hipGetDevice(&h->device));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, h->device));
    h->n_cu = prop.multiProcessorCount;
    for (auto &e : h->ev) HIPCHK(hipEventCreate(&e));
    const size_t tbytes = (size_t)K * K * K * S * 4;
    HIPCHK(hipMalloc(&h->d_table, tbytes));
    {
        int rc = fill_table();
        if (rc) return rc;
    }
    if (h->max_finite >= 0 && (long long)K * h->max_finite >= (1ll << 30))
        return fail(ALPA_DP_EOVERFLOW, "K * largest finite latency >= 2^30");
    h->key_bits_table = bits_for((uint32_t)(h->max_finite + 1));
    h->n_table_keys = K * (K * (K + 1) / 2) * S;
    HIPCHK(hipMalloc(&h->d_sizes, (size_t)S * 4));
    HIPCHK(hipMemcpyAsync(h->d_sizes, sizes.data(), (size_t)S * 4, hipMemcpyHostToDevice,
                          h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));      // `sizes` may go away after the return
    HIPCHK(hipMalloc(&h->pb.hist, (SORT_RADIX * SORT_SLICES + SORT_RADIX) * 4));   // counts + totals
    HIPCHK(hipMalloc(&h->d_ncount, 2 * 4));
    HIPCHK(hipMalloc(&h->d_state, sizeof(SolveState)));
    HIPCHK(hipMemsetAsync(h->d_state, 0, sizeof(SolveState), h->stream));
    HIPCHK(hipMalloc(&h->d_tmpFS, 4 * 4));
    HIPCHK(hipMalloc(&h->d_plan_tmp, sizeof(alpa_plan_t)));
    HIPCHK(hipMalloc(&h->d_best_plan, sizeof(alpa_plan_t)));
    HIPCHK(launch_init_best_plan(h->stream, h->d_best_plan));
    const size_t LS = (size_t)(K + 2) * (D + 1);
    HIPCHK(hipMalloc(&h->d_Fall, (size_t)(h->p.Smax + 1) * LS * 4));
    // general kernel: two F layers per resident workgroup, at most 256 MiB in total
    int gg = h->n_cu * 4;
    while (gg > 1 && (size_t)gg * 2 * LS * 4 > (256ull << 20)) gg /= 2;
    h->generic_grid_max = gg;
    HIPCHK(hipMalloc(&h->d_scratch, (size_t)gg * 2 * LS * 4));
    // register/LDS kernel
    // above 64 devices: one candidate per workgroup, the two-window form of the kernel
    h->fast_ok = K <= 128 && D <= 128;
    if (h->fast_ok) {
        h->KP = 16 * ((K + 15) / 16);
        HIPCHK(hipMalloc(&h->d_recs, fast_table_ints(K, S) * 4));
        HIPCHK(hipMalloc(&h->d_gmin, fast_group_min_ints(K, D, S) * 4));
        HIPCHK(launch_repack_fast(h->stream, h->d_table, K, D, S, h->KP, h->d_recs, h->d_gmin));
        for (int nc = 1; nc <= 2; ++nc) {
            int per_cu = fast_kernel_blocks_per_cu(K, nc);
            if (per_cu < 1) return fail(ALPA_DP_EHIP, "fast kernel does not fit on a CU");
            h->fast_per_cu[nc] = per_cu;
            h->fast_grid_max[nc] = h->n_cu * per_cu;
        }
    }
    int rc2 = ensure_candidate_arrays(h, 0);
    if (rc2) return rc2;
    // length of the full candidate list
    rc2 = queue_table_candidates(h);
    if (rc2) return rc2;
    uint32_t nd = 0;
    HIPCHK(hipMemcpyAsync(&nd, h->d_ncount, 4, hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    h->n_distinct = (int)nd;
    return ALPA_DP_OK;
}

template <class FillTable>
static int create_handle(alpa_dp_t **out, int K, int N, int M, int B,
                         const std::vector<int32_t> &sizes, FillTable fill_table_for)
{
    alpa_dp *h = new (std::nothrow) alpa_dp();
    if (!h) return fail(ALPA_DP_ENOMEM, "host allocation failed");
    const int D = N * M;
    h->p = Problem{K, N, M, D, (int)sizes.size(), std::min(K, D), B};
    const int rc = create_on_device(h, sizes, [&]() { return fill_table_for(h); });
    if (rc != ALPA_DP_OK) {
        std::string keep = g_err;
        alpa_dp_destroy(h);
        g_err = keep;
        return rc;
    }
    *out = h;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_create(alpa_dp_t **out, const int32_t *cost_table, int K, int N, int M,
                              int B, const alpa_shape_t *shapes, int num_shapes)
{
    if (!out) return fail(ALPA_DP_EINVAL, "out is null");
    *out = nullptr;
    if (!cost_table || !shapes) return fail(ALPA_DP_EINVAL, "cost_table or shapes is null");
    std::vector<int32_t> sizes;
    int rc = check_problem(K, N, M, B, shapes, num_shapes, sizes);
    if (rc) return rc;
    const int S = num_shapes;
    return create_handle(out, K, N, M, B, sizes, [&](alpa_dp *h) -> int {
        // the range check of the used part of the table (no negative latency; largest finite
        // entry for the overflow proof) is a reduction on the device copy
        int32_t *d_range = nullptr;
        auto body = [&]() -> int {
            HIPCHK(hipMalloc(&d_range, 2 * 4));
            HIPCHK(hipMemcpyAsync(h->d_table, cost_table, (size_t)K * K * K * S * 4,
                                  hipMemcpyHostToDevice, h->stream));
            HIPCHK(launch_table_range(h->stream, h->d_table, K, S, d_range));
            int32_t range[2] = {0, -1};
            HIPCHK(hipMemcpyAsync(range, d_range, sizeof(range), hipMemcpyDeviceToHost, h->stream));
            HIPCHK(hipStreamSynchronize(h->stream));
            if (range[0] < 0) return fail(ALPA_DP_EINVAL, "negative latency in cost_table");
            h->max_finite = range[1];
            return ALPA_DP_OK;
        };
        const int rc2 = body();
        (void)hipFree(d_range);
        return rc2;
    });
}

extern "C" int alpa_dp_create_from_profiles(alpa_dp_t **out, const int32_t *t_l,
                                            const int64_t *mem_stage, const int64_t *mem_act,
                                            int num_options, int64_t mem_device, int K, int N,
                                            int M, int B, const alpa_shape_t *shapes,
                                            int num_shapes)
{
    if (!out) return fail(ALPA_DP_EINVAL, "out is null");
    *out = nullptr;
    if (!t_l || !mem_stage || !mem_act) return fail(ALPA_DP_EINVAL, "a profile array is null");
    if (num_options < 1 || num_options > ALPA_DP_MAX_OPTIONS)
        return fail(ALPA_DP_EINVAL, "num_options out of range");
    if (mem_device < 0) return fail(ALPA_DP_EINVAL, "mem_device is negative");
    std::vector<int32_t> sizes;
    int rc = check_problem(K, N, M, B, shapes, num_shapes, sizes);
    if (rc) return rc;
    const int S = num_shapes, O = num_options;
    // s * mem_act stays far inside int64 when every figure is below 2^52 (s <= 256)
    for (int k = 0; k < K; ++k)
        for (int i = k; i < K; ++i) {
            const size_t e0 = ((size_t)k * K + i) * S * O, cnt = (size_t)S * O;
            for (size_t x = e0; x < e0 + cnt; ++x) {
                if (t_l[x] < 0) return fail(ALPA_DP_EINVAL, "negative latency in t_l");
                if (mem_stage[x] < 0 || mem_act[x] < 0 || mem_stage[x] >= (1ll << 52) ||
                    mem_act[x] >= (1ll << 52))
                    return fail(ALPA_DP_EINVAL, "memory figure outside [0, 2^52)");
            }
        }
    if (mem_device >= (1ll << 62)) return fail(ALPA_DP_EINVAL, "mem_device too large");
    return create_handle(out, K, N, M, B, sizes, [&](alpa_dp *h) -> int {
        const size_t n = (size_t)K * K * S * O;
        int32_t *d_t = nullptr, *d_max = nullptr;
        int64_t *d_ms = nullptr, *d_ma = nullptr;
        auto body = [&]() -> int {
            HIPCHK(hipMalloc(&d_t, n * 4));
            HIPCHK(hipMalloc(&d_ms, n * 8));
            HIPCHK(hipMalloc(&d_ma, n * 8));
            HIPCHK(hipMalloc(&d_max, 4));
            HIPCHK(hipMemcpyAsync(d_t, t_l, n * 4, hipMemcpyHostToDevice, h->stream));
            HIPCHK(hipMemcpyAsync(d_ms, mem_stage, n * 8, hipMemcpyHostToDevice, h->stream));
            HIPCHK(hipMemcpyAsync(d_ma, mem_act, n * 8, hipMemcpyHostToDevice, h->stream));
            HIPCHK(launch_build_table(h->stream, d_t, d_ms, d_ma, K, S, O, mem_device, h->d_table,
                                      d_max));
            int32_t mx = -1;
            HIPCHK(hipMemcpyAsync(&mx, d_max, 4, hipMemcpyDeviceToHost, h->stream));
            HIPCHK(hipStreamSynchronize(h->stream));
            h->max_finite = mx;
            return ALPA_DP_OK;
        };
        const int rc2 = body();
        (void)hipFree(d_t); (void)hipFree(d_ms); (void)hipFree(d_ma); (void)hipFree(d_max);
        return rc2;
    });
}

extern "C" int alpa_dp_restrict_equal_layers(alpa_dp_t *h)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    const int K = h->p.K, D = h->p.D, S = h->p.S;
    HIPCHK(launch_equal_layer_mask(h->stream, h->d_table, K, S));
    if (h->fast_ok) {
        HIPCHK(launch_repack_fast(h->stream, h->d_table, K, D, S, h->KP, h->d_recs, h->d_gmin));
    }
    // the candidate list changes with the table; the running best belonged to the old one
    int rc = queue_table_candidates(h);
    if (rc) return rc;
    uint32_t nd = 0;
    HIPCHK(hipMemcpyAsync(&nd, h->d_ncount, 4, hipMemcpyDeviceToHost, h->stream));
    HIPCHK(launch_init_best_plan(h->stream, h->d_best_plan));
    HIPCHK(hipStreamSynchronize(h->stream));
    h->n_distinct = (int)nd;
    h->any_solve = false;
    h->have_best = false;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_get_table(alpa_dp_t *h, int32_t *out_table)
{
    if (!h || !out_table) return fail(ALPA_DP_EINVAL, "null argument");
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    const size_t bytes = (size_t)h->p.K * h->p.K * h->p.K * h->p.S * 4;
    HIPCHK(hipMemcpyAsync(out_table, h->d_table, bytes, hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_set_stream(alpa_dp_t *h, void *hip_stream)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    HIPCHK(hipStreamSynchronize(h->stream));
    h->stream = (hipStream_t)hip_stream;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_set_B(alpa_dp_t *h, int B)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    if (B < 1) return fail(ALPA_DP_EINVAL, "B must be >= 1");
    if (B == h->p.B) return ALPA_DP_OK;
    // T* of Eq. 4 under different B values do not compare: the running best starts over
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    HIPCHK(launch_init_best_plan(h->stream, h->d_best_plan));
    h->have_best = false;
    h->p.B = B;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_set_tuning(alpa_dp_t *h, int key, int value)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    switch (key) {
    case ALPA_DP_TUNE_CANDIDATES_PER_WG:
        if (value < 0 || value > 2) return fail(ALPA_DP_EINVAL, "candidates per workgroup: 0, 1 or 2");
        h->tune_nc = value;
        return ALPA_DP_OK;
    case ALPA_DP_TUNE_DISTINCT_BY_SORT:
        if (value < 0 || value > 1) return fail(ALPA_DP_EINVAL, "distinct values by sort: 0 or 1");
        h->tune_sort = value;
        return ALPA_DP_OK;
    case ALPA_DP_TUNE_WG_PER_CU:
        if (value < 0) return fail(ALPA_DP_EINVAL, "workgroups per compute unit: >= 0");
        h->tune_wg_per_cu = value;
        for (int nc = 1; nc <= 2; ++nc) {
            const int per_cu = (value >= 1 && value < h->fast_per_cu[nc]) ? value : h->fast_per_cu[nc];
            h->fast_grid_max[nc] = h->n_cu * per_cu;
        }
        return ALPA_DP_OK;
    case ALPA_DP_TUNE_LANE_GROUPS:
        if (value < 0 || value > 64 || (value & (value - 1)) != 0)
            return fail(ALPA_DP_EINVAL, "lane groups: 0 (own choice), 1 (off) or 2, 4, .. 64 groups");
        h->tune_no_groups = value;
        return ALPA_DP_OK;
    case ALPA_DP_TUNE_WORKGROUPS:
        if (value < 0) return fail(ALPA_DP_EINVAL, "workgroups: >= 0");
        h->tune_grid = value;
        return ALPA_DP_OK;
    default:
        return fail(ALPA_DP_EINVAL, "unknown tuning key");
    }
}

extern "C" int alpa_dp_count_candidates(alpa_dp_t *h, int *out_n)
{
    if (!h || !out_n) return fail(ALPA_DP_EINVAL, "null argument");
    *out_n = h->n_distinct;
    return ALPA_DP_OK;
}

// Upper bound, known on the host, of the number of distinct candidates of a solve.
static int candidate_bound(const alpa_dp *h, bool have_list, int n_tmax)
{
    if (have_list) return n_tmax;
    if (n_tmax == 0) return h->n_distinct;
    return std::min(h->n_distinct, n_tmax);
}

// n_B > 0: sweep over the B values in d_sw_B (Eq. 4 and the selection once per value, plans
// to d_sw_plans); otherwise one solve with the handle's B.
static int solve_dev_impl(alpa_dp *h, const int32_t *d_tmax, int n_tmax, unsigned flags,
                          int64_t *d_out_T, alpa_plan_t *d_out_plan, int key_bits, int n_B = 0)
{
    const Problem &p = h->p;
    const bool have_list = d_tmax != nullptr;
    if (n_tmax < 0) return fail(ALPA_DP_EINVAL, "n_tmax < 0");
    if (have_list && n_tmax == 0) return fail(ALPA_DP_EINVAL, "empty candidate list");
    if (!have_list && n_tmax == 1) return fail(ALPA_DP_EINVAL, "fewer than two quantiles");
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    {
        const int rc = ensure_candidate_arrays(h, have_list ? n_tmax : 0);
        if (rc) return rc;
    }
    const int bound = candidate_bound(h, have_list, n_tmax);
    const int prune_sel = (flags & ALPA_DP_PRUNE) ? 1 : 0;
    // Skipping a candidate while the recurrence runs is decided with one B; a sweep
    // evaluates every candidate and applies the early-exit rule per B in the selection.
    const int prune = n_B > 0 ? 0 : prune_sel;
    hipStream_t st = h->stream;

    HIPCHK(hipEventRecord(h->ev[0], st));
    HIPCHK(launch_init_state(st, h->d_state, h->d_chunkmin, bound / PRUNE_CHUNK + 1));
    if (have_list) {
        HIPCHK(hipMemcpyAsync(h->pb.keys[0], d_tmax, (size_t)n_tmax * 4, hipMemcpyDeviceToDevice,
                              st));
        HIPCHK(launch_sort_dedup(st, h->pb, n_tmax, key_bits, /*drop_key=*/-1, h->d_cand,
                                 h->d_ncount + 1));
        HIPCHK(launch_set_candidates(st, h->d_ncount + 1, h->d_state));
        if (d_out_T)
            HIPCHK(launch_rank_lookup(st, d_tmax, n_tmax, h->d_cand, h->d_ncount + 1, h->d_rank));
    } else {
        int rc = queue_table_candidates(h);
        if (rc) return rc;
        HIPCHK(launch_pick_candidates(st, h->d_distinct, h->d_ncount + 0, n_tmax, h->d_cand,
                                      h->d_state, h->cand_cap));
    }
    HIPCHK(hipEventRecord(h->ev[1], st));
    if (bound > 0) {
        const bool fast = h->fast_ok && !(flags & ALPA_DP_GENERIC);
        if (fast) {
            // One candidate per workgroup: seven waves per SIMD and two columns folded into one
            // three-operand minimum, which is faster than two candidates sharing their scalar
            // loads and lanes at four waves per SIMD (workload 4: 4.40 against 4.66 ms); the
            // two-candidate form stays available through the tuning call.
            int nc = 1;
            if (h->tune_nc) nc = h->tune_nc;
            const bool wide = p.D > 64;            // two windows of device counts, one candidate
            if (wide) nc = 2;
            // Small meshes: groups of lanes, each with a candidate of its own: as many groups as
            // the mesh allows (less work in total, and fewer, lonelier workgroups, which on these
            // small problems matters as much: workload 2 takes 0.11 instead of 0.15 ms).  Not for
            // lists so short that every candidate gets a compute unit of its own anyway.
            int group_dp = 0;
            if (p.D <= 32 && nc == 1 && h->tune_no_groups != 1 &&
                (bound > h->n_cu || h->tune_no_groups >= 2)) {
                group_dp = fast_lane_group_width(p.D);
                if (h->tune_no_groups >= 2) group_dp = std::max(group_dp, WAVE / h->tune_no_groups);
            }
            const bool grouped = group_dp != 0;
            const int per_wg = wide ? 1 : (grouped ? WAVE / group_dp : nc);
            const int n_groups = (bound + per_wg - 1) / per_wg;
            const int grid = std::max(
                1, std::min(n_groups, h->tune_grid ? h->tune_grid : h->fast_grid_max[nc]));
            FastArgs fa{p, h->d_recs, h->d_sizes, h->d_cand, &h->d_state->n_cand,
                        &h->d_state->ticket, &h->d_state->wave_relax, h->d_chunkmin, prune,
                        /*descending=*/prune ? 0 : 1, h->d_Fmin, h->d_Sbest, h->cand_cap, nullptr, nullptr, h->d_gmin};
            fa.grouped = group_dp;
            HIPCHK(launch_recurrence_fast(st, fa, (flags & ALPA_DP_COUNT_WORK) ? FAST_MODE_COUNT
                                                                              : FAST_MODE_BATCH,
                                          nc, grid));
        } else {
            const int grid = std::max(1, std::min(bound, h->generic_grid_max));
            HIPCHK(launch_recurrence_generic(st, p, h->d_table, h->d_sizes, h->d_cand,
                                             &h->d_state->n_cand, &h->d_state->ticket,
                                             h->d_chunkmin, prune, h->d_Fmin, h->d_Sbest,
                                             h->d_scratch, 2, grid));
        }
    }
    HIPCHK(hipEventRecord(h->ev[2], st));
    if (n_B > 0) {
        HIPCHK(launch_sweep_epilogue(st, h->d_sw_B, n_B, &h->d_state->n_cand, h->d_cand, h->d_Fmin,
                                     h->d_Sbest, h->d_sw_state, prune_sel, h->d_sw_c, h->d_sw_s));
        if (h->fast_ok && p.D <= 64 && !(flags & ALPA_DP_GENERIC)) {
            const size_t slab = (size_t)(p.Smax + 1) * (size_t)(p.K + 2) * (p.D + 1);
            FastArgs fa{p, h->d_recs, h->d_sizes, h->d_sw_c, h->d_sw_n, h->d_sw_n + 1,
                        &h->d_state->wave_relax, nullptr, 0, 0, h->d_sw_FS,
                        h->d_sw_FS + (n_B + 1), n_B, h->d_sw_Fall, h->d_sw_s, h->d_gmin};
            HIPCHK(launch_recurrence_fast(st, fa, FAST_MODE_PLAN, 1, std::min(n_B, h->n_cu)));
            HIPCHK(launch_plan_walk_many(st, p, h->d_table, h->d_sizes, h->d_sw_state,
                                         h->d_sw_Fall, slab, h->d_sw_plans, n_B));
        } else {
            for (int b = 0; b < n_B; ++b) {        // one slab of layers, reused in stream order
                SolveState *sb = h->d_sw_state + b;
                HIPCHK(launch_plan_layers(st, p, h->d_table, h->d_sizes, h->d_sw_c + b,
                                          &sb->plan_n, h->d_sw_s + b, h->d_Fall));
                HIPCHK(launch_plan_walk_many(st, p, h->d_table, h->d_sizes, sb, h->d_Fall, 0,
                                             h->d_sw_plans + b, 1));
            }
        }
        HIPCHK(hipEventRecord(h->ev[3], st));
        h->any_solve = true;
        h->timed = true;
        return ALPA_DP_OK;
    }
    HIPCHK(launch_epilogue(st, p, h->d_cand, h->d_Fmin, h->d_Sbest, h->d_state, prune_sel, h->d_T));
    if (d_out_T && bound > 0)
        HIPCHK(launch_scatter_T(st, h->d_T, have_list ? h->d_rank : nullptr,
                                have_list ? n_tmax : bound, h->d_state, d_out_T));
    // every layer of the winning candidate (does nothing if there is none), then the walk
    if (h->fast_ok && p.D <= 64 && !(flags & ALPA_DP_GENERIC)) {
        FastArgs fa{p, h->d_recs, h->d_sizes, &h->d_state->best_c,
                    &h->d_state->plan_n, &h->d_state->plan_ticket, &h->d_state->wave_relax,
                    nullptr, 0, 0, h->d_tmpFS, h->d_tmpFS + 2, 1, h->d_Fall, &h->d_state->best_s,
                    h->d_gmin};
        HIPCHK(launch_recurrence_fast(st, fa, FAST_MODE_PLAN, 1, 1));
    } else {
        HIPCHK(launch_plan_layers(st, p, h->d_table, h->d_sizes, &h->d_state->best_c,
                                  &h->d_state->plan_n, &h->d_state->best_s, h->d_Fall));
    }
    HIPCHK(launch_plan_walk(st, p, h->d_table, h->d_sizes, h->d_state, h->d_Fall, h->d_plan_tmp,
                            h->d_best_plan, d_out_plan));
    HIPCHK(hipEventRecord(h->ev[3], st));
    h->any_solve = true;
    h->have_best = true;
    h->timed = true;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_solve_dev(alpa_dp_t *h, const int32_t *d_tmax, int n_tmax, unsigned flags,
                                 int64_t *d_out_T, alpa_plan_t *d_out_plan)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    return solve_dev_impl(h, d_tmax, n_tmax, flags, d_out_T, d_out_plan, 31);
}

// Checks a host candidate list and queues its copy to the device; *d_tmax stays null if
// there is none.
static int stage_host_candidates(alpa_dp *h, const int32_t *tmax, int n_tmax,
                                 const int32_t **d_tmax, int *key_bits)
{
    *d_tmax = nullptr;
    *key_bits = 31;
    if (tmax) {
        if (n_tmax == 0) return fail(ALPA_DP_EINVAL, "empty candidate list");
        int32_t mx = 0;
        for (int j = 0; j < n_tmax; ++j) {
            if (tmax[j] < 0 || tmax[j] == ALPA_DP_INF_I32)
                return fail(ALPA_DP_EINVAL, "candidate out of range");
            mx = std::max(mx, tmax[j]);
        }
        *key_bits = bits_for((uint32_t)mx);
        {
            const int rc = ensure_candidate_arrays(h, n_tmax);
            if (rc) return rc;
        }
        HIPCHK(hipMemcpyAsync(h->d_tmax_stage, tmax, (size_t)n_tmax * 4, hipMemcpyHostToDevice,
                              h->stream));
        *d_tmax = h->d_tmax_stage;
    }
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_solve(alpa_dp_t *h, const int32_t *tmax, int n_tmax, unsigned flags,
                             int64_t *out_T, alpa_plan_t *out_plan)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    if (n_tmax < 0) return fail(ALPA_DP_EINVAL, "n_tmax < 0");
    int key_bits = 31;
    const int32_t *d_tmax = nullptr;
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    {
        int rc = stage_host_candidates(h, tmax, n_tmax, &d_tmax, &key_bits);
        if (rc) return rc;
    }
    const int n_out = candidate_bound(h, tmax != nullptr, n_tmax);
    int rc = solve_dev_impl(h, d_tmax, n_tmax, flags, out_T ? h->d_outT_stage : nullptr,
                            out_plan ? h->d_plan_tmp : nullptr, key_bits);
    if (rc) return rc;
    if (out_T && n_out > 0)
        HIPCHK(hipMemcpyAsync(out_T, h->d_outT_stage, (size_t)n_out * 8, hipMemcpyDeviceToHost,
                              h->stream));
    if (out_plan)
        HIPCHK(hipMemcpyAsync(out_plan, h->d_plan_tmp, sizeof(alpa_plan_t), hipMemcpyDeviceToHost,
                              h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    if (out_plan && out_plan->num_stages < 0)
        return fail(ALPA_DP_EHIP, "internal inconsistency during plan recovery");
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_solve_sweep(alpa_dp_t *h, const int32_t *tmax, int n_tmax, unsigned flags,
                                   const int32_t *B_values, int n_B, alpa_plan_t *out_plans)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    if (n_tmax < 0) return fail(ALPA_DP_EINVAL, "n_tmax < 0");
    if (!B_values || !out_plans) return fail(ALPA_DP_EINVAL, "B_values or out_plans is null");
    if (n_B < 1 || n_B > ALPA_DP_MAX_SWEEP) return fail(ALPA_DP_EINVAL, "n_B out of range");
    for (int b = 0; b < n_B; ++b)
        if (B_values[b] < 1) return fail(ALPA_DP_EINVAL, "B must be >= 1");
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    int key_bits = 31;
    const int32_t *d_tmax = nullptr;
    int rc = stage_host_candidates(h, tmax, n_tmax, &d_tmax, &key_bits);
    if (rc) return rc;
    if (n_B > h->sw_cap) {
        HIPCHK(hipStreamSynchronize(h->stream));
        rc = alloc_sweep_arrays(h, n_B);
        if (rc) return rc;
    }
    const int32_t head[2] = {n_B, 0};
    HIPCHK(hipMemcpyAsync(h->d_sw_n, head, sizeof(head), hipMemcpyHostToDevice, h->stream));
    HIPCHK(hipMemcpyAsync(h->d_sw_B, B_values, (size_t)n_B * 4, hipMemcpyHostToDevice, h->stream));
    rc = solve_dev_impl(h, d_tmax, n_tmax, flags, nullptr, nullptr, key_bits, n_B);
    if (rc) {
        (void)hipStreamSynchronize(h->stream);     // `head` above is read by a queued copy
        return rc;
    }
    HIPCHK(hipMemcpyAsync(out_plans, h->d_sw_plans, (size_t)n_B * sizeof(alpa_plan_t),
                          hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    for (int b = 0; b < n_B; ++b)
        if (out_plans[b].num_stages < 0)
            return fail(ALPA_DP_EHIP, "internal inconsistency during plan recovery");
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_candidates(alpa_dp_t *h, int32_t *out, int cap, int *out_n)
{
    if (!h || !out_n || (cap > 0 && !out)) return fail(ALPA_DP_EINVAL, "null argument");
    if (!h->any_solve) return fail(ALPA_DP_EINVAL, "no solve has been made on this handle");
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    SolveState s;
    HIPCHK(hipMemcpyAsync(&s, h->d_state, sizeof(s), hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    *out_n = s.n_cand;
    const int n = std::min(cap, s.n_cand);
    if (n > 0) {
        HIPCHK(hipMemcpyAsync(out, h->d_cand, (size_t)n * 4, hipMemcpyDeviceToHost, h->stream));
        HIPCHK(hipStreamSynchronize(h->stream));
    }
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_best(alpa_dp_t *h, alpa_plan_t *out_plan)
{
    if (!h || !out_plan) return fail(ALPA_DP_EINVAL, "null argument");
    if (!h->have_best) {
        int rc = alpa_dp_solve(h, nullptr, 0, ALPA_DP_PRUNE, nullptr, nullptr);
        if (rc) return rc;
    }
    int prev = 0;
    HIPCHK(hipGetDevice(&prev));
    if (prev != h->device) HIPCHK(hipSetDevice(h->device));
    struct Restore { int prev, cur; ~Restore() { if (prev != cur) (void)hipSetDevice(prev); } }
        restore{prev, h->device};
    HIPCHK(hipMemcpyAsync(out_plan, h->d_best_plan, sizeof(alpa_plan_t), hipMemcpyDeviceToHost,
                          h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_last_timing(alpa_dp_t *h, float *ms_candidates, float *ms_recurrence,
                                   float *ms_epilogue)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    if (!h->timed) return fail(ALPA_DP_EINVAL, "no solve has been made on this handle");
    HIPCHK(hipEventSynchronize(h->ev[3]));
    float a = 0, b = 0, c = 0;
    HIPCHK(hipEventElapsedTime(&a, h->ev[0], h->ev[1]));
    HIPCHK(hipEventElapsedTime(&b, h->ev[1], h->ev[2]));
    HIPCHK(hipEventElapsedTime(&c, h->ev[2], h->ev[3]));
    if (ms_candidates) *ms_candidates = a;
    if (ms_recurrence) *ms_recurrence = b;
    if (ms_epilogue) *ms_epilogue = c;
    return ALPA_DP_OK;
}

extern "C" int alpa_dp_last_counters(alpa_dp_t *h, int *n_candidates, int64_t *wave_relaxations)
{
    if (!h) return fail(ALPA_DP_EINVAL, "handle is null");
    if (!h->any_solve) return fail(ALPA_DP_EINVAL, "no solve has been made on this handle");
    SolveState s;
    HIPCHK(hipMemcpyAsync(&s, h->d_state, sizeof(s), hipMemcpyDeviceToHost, h->stream));
    HIPCHK(hipStreamSynchronize(h->stream));
    if (n_candidates) *n_candidates = s.n_cand;
    if (wave_relaxations) *wave_relaxations = (int64_t)s.wave_relax;
    return ALPA_DP_OK;
}
