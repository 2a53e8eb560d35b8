/*
 * alpa_dp.h — C ABI of the MI355X (gfx950) stage-slicing dynamic program.
 *
 * The library solves the inter-operator planning problem of Sec. 5.1-5.2:
 * cut K layers into contiguous pipeline stages, give every stage one submesh
 * shape out of a fixed family so that the device counts add up to N*M, and
 * minimise   sum_i t_i + (B - 1) * max_j t_j   (Eq. 2)   by enumerating the
 * bound t_max, minimising the latency sum under "every stage <= t_max" with
 * the recurrence F(s, k, d; t_max) (Eq. 3) and adding (B - 1) * t_max (Eq. 4),
 * as in the dynamic-programming loop of Alg. 1.  Every step runs in HIP
 * kernels on the device the handle was created on; there is no CPU fallback.
 *
 * Conventions
 *   - latencies are int32 microseconds, >= 0; INT32_MAX means +infinity
 *     (stage does not fit in memory, Eq. 5); sums and T* are int64;
 *   - layers are 0-based at this boundary; a stage is [first, last];
 *   - the third table index s is "number of stages from this stage to the last
 *     one, inclusive" (the s of Eq. 3), 1 <= s <= K;
 *   - tie-breaks are fixed so that results are unique: inside Eq. 3 the lowest
 *     last layer, then the lowest shape index; in Eq. 4 the lowest s; over
 *     candidates the lowest t_max;
 *   - the filter of Eq. 3 is  t_intra <= t_max.
 *
 * All functions return ALPA_DP_OK (0) or a negative error code and never throw
 * or abort; alpa_dp_last_error() gives a message for the calling thread's last
 * failure.  An infeasible problem is not an error (T_star = ALPA_DP_INF_I64,
 * num_stages = 0).  A handle may be used by one thread at a time; distinct
 * handles are independent.
 */
#ifndef ALPA_DP_H
#define ALPA_DP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ALPA_DP_MAX_K        256          /* most layers                         */
#define ALPA_DP_MAX_DEVICES  1024         /* largest N*M                         */
#define ALPA_DP_MAX_SHAPES   64           /* most submesh shapes                 */
#define ALPA_DP_INF_I32      INT32_MAX    /* +infinity in cost_table             */
#define ALPA_DP_INF_I64      INT64_MAX    /* infeasible / not evaluated T*       */

#define ALPA_DP_OK            0
#define ALPA_DP_EINVAL       (-1)         /* bad argument                        */
#define ALPA_DP_EOVERFLOW    (-2)         /* K * max finite latency >= 2^30      */
#define ALPA_DP_ENOMEM       (-3)         /* host or device allocation failed    */
#define ALPA_DP_EHIP         (-4)         /* a HIP call failed                   */

/* flags of alpa_dp_solve / alpa_dp_solve_dev */
#define ALPA_DP_PRUNE         1u          /* early pruning of Alg. 1 / Sec. 5.2 opt. #1 */
#define ALPA_DP_COUNT_WORK    4u          /* tally executed work (alpa_dp_last_counters) */
#define ALPA_DP_GENERIC       2u          /* use the general kernel even where the
                                             register/LDS kernel applies         */

typedef struct alpa_dp alpa_dp_t;         /* opaque, owned by the library        */

typedef struct { int32_t n, m; } alpa_shape_t;   /* submesh of n x m devices    */

typedef struct {
    int64_t T_star;                       /* Eq. 2 value; ALPA_DP_INF_I64 if none      */
    int32_t t_max;                        /* winning candidate (us); 0 if none         */
    int32_t num_stages;                   /* stages of the plan; 0 if none             */
    int32_t n_evaluated;                  /* candidates processed before the pruning
                                             break (= number of distinct candidates
                                             when pruning is off)                      */
    int32_t first_layer[ALPA_DP_MAX_K + 1]; /* stage p (pipeline order) holds layers
                                             [first_layer[p], first_layer[p+1])        */
    int32_t shape_idx[ALPA_DP_MAX_K];     /* index into shapes[] for stage p           */
} alpa_plan_t;

/*
 * Problem statement of Sec. 5.1 (operators o_1..o_K, cluster mesh N x M, B
 * microbatches) plus the t_intra table of Sec. 5.2 / Alg. 1 ("costs of different
 * stage-mesh pairs").
 *
 *   cost_table  HOST pointer, read during the call only (the library keeps its own
 *               device copies in the layouts its kernels want).  C order
 *               [s-1][k][i][q], extents K x K x K x num_shapes; k / i = first / last
 *               layer of the stage; entries with i < k are ignored.
 *   shapes      HOST pointer, read during the call only.  Every shape must belong to
 *               the family of Sec. 5.2: (1, 2^p) with 2^p <= M, or (n, M) with
 *               2 <= n <= N; M must be a power of two (Appendix A).  The order
 *               defines the shape index used in tie-breaks; duplicates are allowed.
 *   *out        receives the handle; destroy with alpa_dp_destroy.
 *
 * Errors: EINVAL (null pointer, K < 1 or > ALPA_DP_MAX_K, N*M > ALPA_DP_MAX_DEVICES,
 * B < 1, num_shapes < 1 or > ALPA_DP_MAX_SHAPES, shape outside the family, negative
 * latency), EOVERFLOW (K * largest finite latency >= 2^30: the kernels add in int32),
 * ENOMEM, EHIP.  The device is the calling thread's current HIP device; work is
 * queued on the null stream until alpa_dp_set_stream is called.
 */
int alpa_dp_create(alpa_dp_t **out, const int32_t *cost_table,
                   int K, int N, int M, int B,
                   const alpa_shape_t *shapes, int num_shapes);

/*
 * Same handle, with the t_intra table built on the device from profiled options
 * (Sec. 5.2, the paragraph that defines t_intra, Eq. 5, and the intra-op loop nest of
 * Alg. 1): for stage (k..i), submesh shape q and s stages from this one to the last,
 *   t_intra = min over options o with mem_stage + s * mem_act <= mem_device of t_l,
 * +infinity (ALPA_DP_INF_I32) if no option fits; s = 1..K.
 *
 *   t_l        HOST int32 [k][i][q][o] (C order, extents K x K x num_shapes x
 *              num_options), microseconds; ALPA_DP_INF_I32 = the option does not exist.
 *              An option is a logical mesh shape with n_q * m_q devices combined with
 *              an intra-op option.  Entries with i < k are ignored.
 *   mem_stage  HOST int64, same layout: bytes per device to run the stage.
 *   mem_act    HOST int64, same layout: bytes per device per stored set of activations.
 *   mem_device bytes per device.
 *   The other arguments are those of alpa_dp_create.  All arrays are read during the
 *   call only.
 *
 * Errors: those of alpa_dp_create, and EINVAL for num_options < 1 or >
 * ALPA_DP_MAX_OPTIONS, a negative latency, a memory figure outside [0, 2^52), or
 * mem_device outside [0, 2^62).
 */
#define ALPA_DP_MAX_OPTIONS 32
int alpa_dp_create_from_profiles(alpa_dp_t **out, const int32_t *t_l,
                                 const int64_t *mem_stage, const int64_t *mem_act,
                                 int num_options, int64_t mem_device,
                                 int K, int N, int M, int B,
                                 const alpa_shape_t *shapes, int num_shapes);

/*
 * "Equal layer" variant of the ablation study (Sec. 8.3): restricts the handle, for good, to
 * plans whose stages all have the same number of layers.  With s stages from first layer k
 * to the last one that number is (K - k) / s, so table entry (s, k, i) is kept iff s divides
 * K - k and i - k + 1 == (K - k) / s; every other entry becomes +infinity.  The candidate
 * count (alpa_dp_count_candidates) changes with it and the running best of alpa_dp_best is
 * reset.  Blocking.
 */
int alpa_dp_restrict_equal_layers(alpa_dp_t *h);

/* Copies the handle's table, C order [s-1][k][i][q] (K x K x K x num_shapes int32), to
 * the HOST array out_table.  Blocking. */
int alpa_dp_get_table(alpa_dp_t *h, int32_t *out_table);

/* Queue all later work of this handle on `hip_stream` (a hipStream_t; e.g. the
 * cuda_stream field of a torch.cuda.Stream).  The caller keeps the stream alive. */
int alpa_dp_set_stream(alpa_dp_t *h, void *hip_stream);

/* Change B (Sec. 7: B is a hyper-parameter searched by enumeration).  B >= 1.  T* of Eq. 4
 * under different B do not compare, so a change of B resets the running best of alpa_dp_best
 * (which is then the best over the solves made since).  Errors: EINVAL, EHIP. */
int alpa_dp_set_B(alpa_dp_t *h, int B);

/*
 * Tuning of the launch shape; cites no passage of the paper because no result depends on it
 * (the parity tests run every setting against the same oracle values).  value 0 restores the
 * library's own choice.  Errors: EINVAL (null handle, unknown key, value out of range).
 */
#define ALPA_DP_TUNE_CANDIDATES_PER_WG 1  /* 1 or 2 t_max candidates per workgroup of the
                                             register/LDS kernel (own choice: 1)                 */
#define ALPA_DP_TUNE_DISTINCT_BY_SORT  2  /* 1: distinct table values by the radix sort also where
                                             the presence bitmap applies                        */
#define ALPA_DP_TUNE_WG_PER_CU         3  /* upper bound on resident workgroups per compute unit */
#define ALPA_DP_TUNE_LANE_GROUPS        5  /* meshes of up to 32 devices: 1 = do not cut the wave
                                             into lane groups with a candidate each; 2, 4, .. 64
                                             = that many groups (at most 64 / devices rounded up
                                             to a power of two)                                 */
#define ALPA_DP_TUNE_WORKGROUPS        4  /* workgroups launched by the register/LDS kernel (own
                                             choice: as many as are resident at once; more than
                                             that and each takes fewer candidate groups)        */
int alpa_dp_set_tuning(alpa_dp_t *h, int key, int value);

/* Number of distinct finite values of the table (entries with i >= k): the length
 * of Alg. 1's "SortedAndFilter(t_intra, epsilon)" list for integer latencies and
 * epsilon = 1 us.  Computed on the device at create time. */
int alpa_dp_count_candidates(alpa_dp_t *h, int *out_n);

/*
 * The dynamic-programming loop of Alg. 1 over a list of t_max candidates, blocking.
 *
 *   tmax     HOST pointer to n_tmax candidates in any order, duplicates allowed
 *            (sorted and deduplicated on the device), each in [0, INT32_MAX); or NULL:
 *            then the candidates are the distinct finite table values, ascending —
 *            all of them if n_tmax == 0, else n_tmax evenly spaced quantiles
 *            v[(j * (n - 1)) / (n_tmax - 1)] (all if there are no more than n_tmax;
 *            n_tmax >= 2).
 *   flags    ALPA_DP_PRUNE: stop at the first candidate (ascending) with
 *            B * t_max >= best T* so far, exactly as the sequential loop would; the
 *            remaining candidates report ALPA_DP_INF_I64.
 *   out_T    HOST pointer or NULL.  tmax != NULL: n_tmax values, out_T[j] = T*(tmax[j])
 *            of Eq. 4 in the caller's order (duplicates get equal values).
 *            tmax == NULL: one value per candidate in ascending candidate order
 *            (alpa_dp_count_candidates() values, or min(that, n_tmax)).
 *   out_plan HOST pointer or NULL: best plan of this call.
 *
 * Errors: EINVAL (null handle, n_tmax < 0, n_tmax == 0 with tmax != NULL, n_tmax == 1
 * with tmax == NULL, candidate out of range), ENOMEM, EHIP.
 */
int alpa_dp_solve(alpa_dp_t *h, const int32_t *tmax, int n_tmax, unsigned flags,
                  int64_t *out_T, alpa_plan_t *out_plan);

/*
 * Same computation with DEVICE pointers, asynchronous on the handle's stream: nothing
 * is copied to or from the host and the call returns once the work is queued.
 * d_tmax (or NULL), d_out_T (or NULL) and d_out_plan (or NULL) are device pointers
 * with the sizes given for alpa_dp_solve; they must stay valid until the stream has
 * run the work.  Candidates are not range-checked (values outside [0, INT32_MAX) give
 * T* = ALPA_DP_INF_I64 or unfiltered results for that candidate, never a fault).
 */
int alpa_dp_solve_dev(alpa_dp_t *h, const int32_t *d_tmax, int n_tmax, unsigned flags,
                      int64_t *d_out_T, alpa_plan_t *d_out_plan);

/*
 * Sweep over the number of microbatches (Sec. 5.2: B is a hyper-parameter found by
 * enumeration).  F of Eq. 3 does not depend on B, so the recurrence runs once for the
 * candidate list and Eq. 4 plus the selection run once per B value.
 *
 *   tmax, n_tmax  as for alpa_dp_solve (HOST pointer or NULL).
 *   flags     ALPA_DP_GENERIC as for alpa_dp_solve.  ALPA_DP_PRUNE: every candidate is
 *             still evaluated (the early exit of Alg. 1 depends on B); the rule is applied
 *             per B value afterwards, so that out_plans[b].n_evaluated and every other
 *             field equal those of alpa_dp_solve with B = B_values[b] and the same flags.
 *   B_values  HOST array of n_B values, each >= 1, 1 <= n_B <= ALPA_DP_MAX_SWEEP.
 *   out_plans HOST array of n_B plans, caller-owned; out_plans[b] is the best plan for
 *             B_values[b] (num_stages == 0 and T_star == ALPA_DP_INF_I64 if infeasible).
 *
 * The handle's own B and the running best of alpa_dp_best() are not touched.  Blocking.
 * On the first call (and when n_B grows) device memory for n_B sets of layers is
 * allocated: n_B * (min(K, N*M) + 1) * (K + 2) * (N*M + 1) * 4 bytes when K <= 128 and
 * N*M <= 64 (one set, reused, otherwise).  Errors: EINVAL (null pointers, n_B or a B value
 * out of range, and the candidate-list errors of alpa_dp_solve), ENOMEM, EHIP.
 */
#define ALPA_DP_MAX_SWEEP 256
int alpa_dp_solve_sweep(alpa_dp_t *h, const int32_t *tmax, int n_tmax, unsigned flags,
                        const int32_t *B_values, int n_B, alpa_plan_t *out_plans);

/* Ascending distinct candidate list of the last solve on this handle: copies at most
 * `cap` values to the HOST array `out` and stores the count in *out_n.  Blocking. */
int alpa_dp_candidates(alpa_dp_t *h, int32_t *out, int cap, int *out_n);

/* Best plan over every alpa_dp_solve / alpa_dp_solve_dev made on the handle with its present
 * table and B (lowest T*, then lowest t_max); sweeps do not count.  If there was none, runs
 * alpa_dp_solve(h, NULL, 0, ALPA_DP_PRUNE, NULL, out_plan) first ("the minimal pipeline
 * execution latency T*" that Alg. 1 outputs).  Blocking. */
int alpa_dp_best(alpa_dp_t *h, alpa_plan_t *out_plan);

/* Device time of the phases of the last solve, from HIP events recorded on the
 * handle's stream: candidate preparation (sort / dedup / quantiles), the recurrence
 * kernel of Eq. 3, and Eq. 4 + best selection + plan recovery.  Blocking.  Any
 * pointer may be NULL. */
int alpa_dp_last_timing(alpa_dp_t *h, float *ms_candidates, float *ms_recurrence,
                        float *ms_epilogue);

/* Counters of the last solve: number of distinct candidates, and the number of
 * wave-level relaxation instructions' worth of work the recurrence kernel issued
 * (64-lane add+min pairs), for the benchmark's executed-work figure.  Blocking. */
int alpa_dp_last_counters(alpa_dp_t *h, int *n_candidates, int64_t *wave_relaxations);

void alpa_dp_destroy(alpa_dp_t *h);

/* Message of the calling thread's last failed call ("" if none).  Never NULL. */
const char *alpa_dp_last_error(void);

/*
 * Operator clustering (Sec. 5.2, performance optimisation #2, Eq. 6): cut the operators
 * o_1..o_K (topological order) into L consecutive layers so that the largest amount of data
 * any layer receives from earlier operators is smallest,
 *   G(k, r) = min over 1 <= i <= k with FLOP(o_i..o_k) <= (1 + delta) FLOP_total / L
 *             of max{G(i-1, r-1), C(i, k)},
 * ties going to the smaller sum of squared per-layer FLOP (the lower variance), then to the
 * smaller i, cell by cell.  Stateless; runs on the calling thread's current device, null
 * stream; blocking.  All pointers are HOST pointers, read / written during the call only.
 *
 *   flop          int32 [K], >= 0, any unit; total < 2^31 and total * L < 2^42.
 *   edge_src/dst  int32 [num_edges], 0-based operators, src < dst; parallel edges add up.
 *   edge_bytes    int64 [num_edges], >= 0, sum < 2^62.
 *   delta_ppm     delta in parts per million, 0..10^9; the FLOP condition is evaluated in
 *                 integers: FLOP(i..k) * L * 10^6 <= (10^6 + delta_ppm) * total.
 *   *out_comm     G(K, L), or ALPA_DP_INF_I64 if no clustering satisfies the FLOP bound
 *                 (then *out_sumsq = 0 and out_first_op[] = -1).
 *   *out_sumsq    sum of squared per-layer FLOP of the clustering returned.
 *   out_first_op  int32 [L + 1]: layer r = operators [out_first_op[r], out_first_op[r+1]).
 *   out_ms        NULL, or receives the device time of the kernels (HIP events).
 *
 * Errors: EINVAL (null pointer, K or L outside 1..ALPA_CLUSTER_MAX_OPS, bad edge, negative
 * figure, delta_ppm out of range), EOVERFLOW (the limits above), ENOMEM (8 K^2 + 4 L K bytes
 * of device memory are needed), EHIP.
 */
#define ALPA_CLUSTER_MAX_OPS 4096
int alpa_cluster_layers(const int32_t *flop, int K, const int32_t *edge_src,
                        const int32_t *edge_dst, const int64_t *edge_bytes, int num_edges,
                        int L, int delta_ppm, int64_t *out_comm, int64_t *out_sumsq,
                        int32_t *out_first_op, float *out_ms);

/*
 * The same clustering with the tie-break of Eq. 6's closing sentence ("if there are multiple
 * solutions with the same communication cost, choose the one with the most uniform structure
 * by also minimising the variance of per-layer FLOP") taken over whole clusterings instead of
 * cell by cell: *out_comm is the same G(K, L); *out_sumsq is the smallest sum of squared
 * per-layer FLOP among ALL clusterings that reach it (never larger than alpa_cluster_layers's),
 * and out_first_op is that clustering (among several, the one whose last layer starts
 * earliest, then whose last but one does, and so on).  Two runs of the recurrence: G alone,
 * then W(k, r) = min over i with the FLOP bound and C(i, k) <= G(K, L) of
 * W(i-1, r-1) + FLOP(o_i..o_k)^2.  Arguments, limits and errors as for alpa_cluster_layers.
 */
int alpa_cluster_layers_exact(const int32_t *flop, int K, const int32_t *edge_src,
                              const int32_t *edge_dst, const int64_t *edge_bytes, int num_edges,
                              int L, int delta_ppm, int64_t *out_comm, int64_t *out_sumsq,
                              int32_t *out_first_op, float *out_ms);

/*
 * alpa_cluster_layers for callers that cannot allocate device memory or wait: code recorded into
 * a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same computation and
 * results; inputs and outputs are DEVICE pointers owned by the caller, the call only queues
 * kernels on `hip_stream` (a hipStream_t, NULL = the null stream) and returns; it calls no
 * hipMalloc / hipFree, copies nothing and does not synchronise.  The work memory is a fixed
 * array in the library's device image (about 3.2 MB per device, held until the process ends),
 * which limits K and L to ALPA_CLUSTER_STATIC_MAX_OPS.
 *
 *   d_flop, d_edge_src, d_edge_dst, d_edge_bytes   as for alpa_cluster_layers, device memory.
 *   d_out           int64 [3]: G(K, L) (ALPA_DP_INF_I64 if none), sum of squared per-layer
 *                   FLOP, and the status of the argument checks that alpa_cluster_layers makes
 *                   on the host and this call makes on the device: 0, ALPA_DP_EINVAL (negative
 *                   figure, bad edge) or ALPA_DP_EOVERFLOW; if not 0 the other outputs are
 *                   those of "no clustering" (INF, 0, -1 ...).  A bad edge is never written.
 *   d_out_first_op  int32 [L + 1].
 * All calls on one device share the one work array: calls that may run at the same time on a
 * device (different streams, different threads) race; serialise them.  Results are valid once
 * the stream has run the work; the input arrays must stay unchanged until then.
 *
 * Errors (returned at once, nothing queued): EINVAL (null pointer, K or L < 1 or above
 * ALPA_CLUSTER_STATIC_MAX_OPS, num_edges < 0, delta_ppm out of range), EHIP.
 */
#define ALPA_CLUSTER_STATIC_MAX_OPS 512
int alpa_cluster_layers_static(const int32_t *d_flop, int K, const int32_t *d_edge_src,
                               const int32_t *d_edge_dst, const int64_t *d_edge_bytes,
                               int num_edges, int L, int delta_ppm, int64_t *d_out,
                               int32_t *d_out_first_op, void *hip_stream);

/*
 * Physical placement of the submeshes a plan chose (Sec. 5.2: devices go to larger submeshes
 * first, then to smaller ones, and neighbouring stages of one shape are put next to each other;
 * Appendix A shows the shapes always cover the mesh, and the construction follows its proof).
 * Host-only (no device work), stateless.
 *
 *   stage_shapes  HOST array of num_stages (n, m) in pipeline order (shapes[plan.shape_idx[p]]),
 *                 each from the family of Sec. 5.2, device counts adding up to N * M.
 *   out_row/col   HOST int32 [num_stages]: stage p owns rows [row, row + n) x columns
 *                 [col, col + m) of the N x M mesh (device id = row * M + col).
 * Order: device count descending, equal counts in pipeline order; positions in row-major order.
 *
 * Errors: EINVAL (null pointer, sizes out of range, M not a power of two, a shape outside the
 * family, device counts not adding up).
 */
int alpa_place_submeshes(int N, int M, const alpa_shape_t *stage_shapes, int num_stages,
                         int32_t *out_row, int32_t *out_col);

/*
 * Measurement aid, outside the method's boundary (no step of the paper): sustained rate of the recurrence's two vector instructions (int32 add with a
 * scalar operand, signed min) from a register-only kernel at full occupancy on the current
 * device, in lane-operations per second, to set beside the nominal peak (compute units x 64
 * lanes x clock).  Blocking, about 50 ms.  Errors: EINVAL (null pointer), EHIP.
 */
int alpa_dp_measure_valu_peak(double *out_lane_ops_per_s);

#ifdef __cplusplus
}
#endif
#endif /* ALPA_DP_H */
