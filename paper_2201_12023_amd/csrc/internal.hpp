// Internal declarations shared by the translation units of libalpa_dp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>

namespace alpa {

// Device-side +infinity.  Finite sums stay below it (checked at create: K * max finite
// latency < 2^30) and INF + INF = 2^31 - 2 still fits in int32, so "never add to
// infinity" becomes "add, then anything >= DEV_INF is infinity".
constexpr int32_t DEV_INF = (1 << 30) - 1;
constexpr int64_t INF_I64 = INT64_MAX;
constexpr int32_t INF_I32 = INT32_MAX;

constexpr int WAVE = 64;
constexpr int PRUNE_CHUNK = 64;          // candidates per published running-minimum slot

// Result block of one solve, in device memory.
struct SolveState {
    int32_t n_cand;          // distinct candidates of this solve
    int32_t ticket;          // next candidate index to hand out (recurrence kernel)
    int32_t n_processed;     // prefix length after the exact pruning rule
    int32_t best_idx;        // index of the winning candidate, -1 if none
    int64_t best_T;          // its T*
    int32_t best_c;          // its t_max
    int32_t best_s;          // its number of stages
    unsigned long long wave_relax;   // executed 64-lane relaxations (instrumented runs)
    int32_t n_distinct;      // distinct finite table values seen by candidate preparation
    int32_t plan_n;          // 1 if a plan is to be recovered (a feasible winner exists)
    int32_t plan_ticket;     // ticket counter of the plan-recovery run
    int32_t pad;
};

struct Problem {
    int K, N, M, D, S, Smax, B;
};

// ---- wave-level reductions (DPP inside rows of 16, ds_swizzle across 16, bpermute across 32)

template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}

// xor-16 inside each half of the wave: ds_swizzle bit mode (and 0x1f, or 0, xor 0x10)
__device__ __forceinline__ int swz_xor16(int v)
{
    return __builtin_amdgcn_ds_swizzle(v, 0x401F);
}

__device__ __forceinline__ int xor32(int v)
{
    return __shfl_xor(v, 32, 64);
}

// min over the 64 lanes, result in every lane
__device__ __forceinline__ int wave_min_i32(int v)
{
    v = min(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    v = min(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    v = min(v, dpp_mov<0x141>(v));   // row_half_mirror
    v = min(v, dpp_mov<0x140>(v));   // row_mirror
    v = min(v, swz_xor16(v));
    v = min(v, xor32(v));
    return v;
}

__device__ __forceinline__ int64_t i64_from(int lo, int hi)
{
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

__device__ __forceinline__ int lo32(int64_t v) { return (int)(uint32_t)(uint64_t)v; }
__device__ __forceinline__ int hi32(int64_t v) { return (int)((uint64_t)v >> 32); }

template <int CTRL>
__device__ __forceinline__ int64_t dpp_mov64(int64_t v)
{
    return i64_from(dpp_mov<CTRL>(lo32(v)), dpp_mov<CTRL>(hi32(v)));
}

__device__ __forceinline__ int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }

__device__ __forceinline__ int64_t wave_min_i64(int64_t v)
{
    v = min64(v, dpp_mov64<0xB1>(v));
    v = min64(v, dpp_mov64<0x4E>(v));
    v = min64(v, dpp_mov64<0x141>(v));
    v = min64(v, dpp_mov64<0x140>(v));
    v = min64(v, i64_from(swz_xor16(lo32(v)), swz_xor16(hi32(v))));
    v = min64(v, i64_from(xor32(lo32(v)), xor32(hi32(v))));
    return v;
}

// inclusive prefix minimum over the 64 lanes (lane l gets min of lanes 0..l)
__device__ __forceinline__ int64_t wave_prefix_min_i64(int64_t v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int lo = __shfl_up(lo32(v), off, 64);
        const int hi = __shfl_up(hi32(v), off, 64);
        const int64_t o = i64_from(lo, hi);
        if (lane >= off) v = min64(v, o);
    }
    return v;
}

// ---- host-side launchers (callers validate sizes first; none of these synchronises)

constexpr int SORT_SLICES = 1024;        // one-wave slices of the radix sort
constexpr int SORT_RADIX = 256;          // 8-bit digits

struct PrepBuffers {
    int32_t *keys[2];        // [cap] each
    uint32_t *hist;          // [SORT_RADIX * SORT_SLICES] slice counts + [SORT_RADIX] digit totals
    uint32_t *block_cnt;     // [cap / 4096 + 2]
    int cap;
};

hipError_t launch_gather_table_values(hipStream_t st, const int32_t *table, int K, int S,
                                      int32_t inf_key, int32_t *out_keys);
hipError_t launch_sort_dedup(hipStream_t st, PrepBuffers &pb, int n, int key_bits,
                             int32_t drop_key, int32_t *out_unique, uint32_t *out_n_unique);
// values below this many bits' worth go through the presence bitmap instead of the sort
constexpr int32_t DISTINCT_BITMAP_MAX = 1 << 19;
hipError_t launch_distinct_by_bitmap(hipStream_t st, const int32_t *table, int K, int S,
                                     int32_t max_value, uint32_t *work, int32_t *out_unique,
                                     uint32_t *out_n_unique);
size_t distinct_bitmap_words(int32_t max_value);
hipError_t launch_pick_candidates(hipStream_t st, const int32_t *distinct,
                                  const uint32_t *n_distinct, int n_quantiles, int32_t *cand,
                                  SolveState *state, int cap);
hipError_t launch_set_candidates(hipStream_t st, const uint32_t *n_unique, SolveState *state);
hipError_t launch_rank_lookup(hipStream_t st, const int32_t *tmax, int n, const int32_t *unique,
                              const uint32_t *n_unique, int32_t *rank_of_orig);

// table[s-1][k][i][q] from profiled options [k][i][q][o]; *max_finite = largest finite entry
// (-1 if none).  O * 1 KiB of LDS per block: O <= 32.
hipError_t launch_build_table(hipStream_t st, const int32_t *t_l, const int64_t *mem_stage,
                              const int64_t *mem_act, int K, int S, int O, int64_t mem_device,
                              int32_t *table, int32_t *max_finite);

// out[0] = smallest, out[1] = largest finite entry (-1 if none) of the used part of a table
hipError_t launch_table_range(hipStream_t st, const int32_t *table, int K, int S, int32_t *out);

hipError_t launch_valu_peak(hipStream_t st, int grid, int iters, int32_t *sink);
hipError_t launch_equal_layer_mask(hipStream_t st, int32_t *table, int K, int S);

hipError_t launch_repack_fast(hipStream_t st, const int32_t *table, int K, int D, int S, int KP,
                              int32_t *recs, int32_t *group_min);
size_t fast_table_ints(int K, int S);    // size of the column-record array, padding included
int fast_group_min_stages(int K, int D);        // stage counts the early-stop table spans
size_t fast_group_min_ints(int K, int D, int S);   // size of the early-stop table

hipError_t launch_recurrence_generic(hipStream_t st, const Problem &p, const int32_t *table,
                                     const int32_t *sizes, const int32_t *cand,
                                     const int32_t *n_cand_p, int32_t *ticket, int64_t *chunk_min,
                                     int prune, int32_t *Fmin, int32_t *Sbest, int32_t *scratch,
                                     int n_layers, int grid);
struct FastArgs {
    Problem p;
    const int32_t *recs, *sizes, *cand, *n_cand_p;
    int32_t *ticket;
    unsigned long long *wave_relax;
    int64_t *chunk_min;
    int prune, descending;
    int32_t *Fmin, *Sbest;
    int dummy_idx;           // spare slot of Fmin / Sbest for the waves that own no result
    // plan mode only: candidate j dumps its layers to F_all + j * (Smax+1) * (K+2)*(D+1) and
    // stops at layer s_top_p[j], the winner's number of stages (device memory)
    int32_t *F_all;
    const int32_t *s_top_p;
    const int32_t *group_min;   // early-stop table (launch_repack_fast)
    // batch modes, at most 32 devices, one-candidate form: 0, or the width DP of the lane groups
    // (a power of two, D <= DP <= 32): 64 / DP candidates per workgroup
    int grouped = 0;
};
// narrowest lane group that holds a mesh of D <= 32 devices
inline int fast_lane_group_width(int D)
{
    int dp = 1;
    while (dp < D) dp <<= 1;
    return dp;
}
enum { FAST_MODE_BATCH = 0, FAST_MODE_COUNT = 1, FAST_MODE_PLAN = 2 };
hipError_t launch_recurrence_fast(hipStream_t st, const FastArgs &a, int mode, int nc, int grid);
int fast_kernel_blocks_per_cu(int K, int nc);
// the instances for 65-128 layers (kernels_fast_deep.hip)
hipError_t launch_recurrence_fast_deep(hipStream_t st, const FastArgs &a, int mode, int nc, int grid);
int fast_kernel_blocks_per_cu_deep(int K, int nc);

// plan recovery of one candidate, a launch per layer (general sizes)
hipError_t launch_plan_layers(hipStream_t st, const Problem &p, const int32_t *table,
                              const int32_t *sizes, const int32_t *c_p, const int32_t *n_p,
                              const int32_t *s_top_p, int32_t *F_all);
hipError_t launch_epilogue(hipStream_t st, const Problem &p, const int32_t *cand,
                           const int32_t *Fmin, const int32_t *Sbest, SolveState *state, int prune,
                           int64_t *T);
hipError_t launch_scatter_T(hipStream_t st, const int64_t *T, const int32_t *rank_of_orig,
                            int n_orig, const SolveState *state, int64_t *out_T);
hipError_t launch_plan_walk(hipStream_t st, const Problem &p, const int32_t *table,
                            const int32_t *sizes, SolveState *state, const int32_t *F_all,
                            void *plan_tmp, void *best_plan, void *plan_out);
// sweep over B: one block per B value
hipError_t launch_sweep_epilogue(hipStream_t st, const int32_t *B_vals, int n_B,
                                 const int32_t *n_cand_p, const int32_t *cand,
                                 const int32_t *Fmin, const int32_t *Sbest, SolveState *states,
                                 int prune, int32_t *win_c, int32_t *win_s);
hipError_t launch_plan_walk_many(hipStream_t st, const Problem &p, const int32_t *table,
                                 const int32_t *sizes, SolveState *states, const int32_t *F_all,
                                 size_t slab, void *plans, int n);
hipError_t launch_init_state(hipStream_t st, SolveState *state, int64_t *chunk_min, int n_chunks);
hipError_t launch_init_best_plan(hipStream_t st, void *best_plan);

// operator clustering (Eq. 6); buffers: Ct [K*K], chunk [cluster_chunk_rows(K)*K], pf [K+1],
// GV [4*(K+1)] (int64), arg [L*(K+1)], out [2] (G, V), first_op [L+1].  ctl == nullptr: the
// caller has checked the inputs and passes the FLOP bound `cap`.  ctl != nullptr ([2] int64):
// the inputs are checked and the bound is computed from delta_ppm on the device, out is [3]
// (G, V, status) and `cap` is ignored.  exact != 0 (host-checked inputs only): a second run of
// the recurrence minimises V over every clustering that reaches G(K, L).
hipError_t launch_cluster(hipStream_t st, const int32_t *flop, const int32_t *src,
                          const int32_t *dst, const int64_t *nbytes, int E, int K, int L,
                          int64_t cap, int64_t *Ct, int64_t *chunk, int64_t *pf, int64_t *GV,
                          int32_t *arg, int64_t *out, int32_t *first_op, int64_t *ctl = nullptr,
                          int delta_ppm = 0, int exact = 0);
size_t cluster_chunk_rows(int K);

}  // namespace alpa
