/*
 * CPU oracle for the stage-slicing dynamic program of the inter-operator pass.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the method computes, written from the paper; only tests,
 * the smoke check and the benchmark's cpu-baseline leg may call it.  It shares
 * no code, header, table or helper with the HIP library.
 *
 * What is followed:
 *   - Eq. 2 (Sec. 5.1): T* = min over slicings and submesh choices of
 *       sum_i t_i + (B - 1) * max_j t_j.
 *   - Eq. 3 (Sec. 5.2): F(s, k, d; t_max) = min over k <= i <= K and shapes q
 *       with a_q <= d and t_intra(k..i, q, s) <= t_max of
 *       t_intra(k..i, q, s) + F(s - 1, i + 1, d - a_q; t_max),  F(0, K+1, 0) = 0.
 *   - Eq. 4: T*(t_max) = min_s F(s, first layer, N*M; t_max) + (B - 1) * t_max.
 *   - Alg. 1, the "inter-op dynamic programming" loop: candidates ascending,
 *     stop when B * t_max >= best T*, keep T*(t_max) when strictly smaller.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - the filter is "<= t_max" (Eq. 3), not the "<" of the running text;
 *   - Eq. 4's "F(s, 0, ...)" means the first layer (1-based: F(s, 1, N*M));
 *   - s is only a table index here and runs 1..min(K, N*M) (more stages than
 *     layers or devices can never be finite);
 *   - tie-breaks: in Eq. 3 the lowest i, then the lowest shape index; in Eq. 4
 *     the lowest s; over candidates the lowest t_max (strict "<" of Alg. 1);
 *   - "sorted and filtered with epsilon": latencies are integer microseconds
 *     and epsilon = 1 us, so this is ascending order without duplicates;
 *   - +infinity is never added to: a term with an infinite operand is skipped;
 *   - quantile candidates: with v[0..n-1] the ascending distinct finite values,
 *     take all if n <= Q, else v[(j * (n - 1)) / (Q - 1)], j = 0..Q-1.
 *
 * Arithmetic: table entries int32 microseconds, all sums int64.
 * Table layout: C order [s-1][k][i][q], extents K x K x K x S, k / i 0-based
 * first / last layer of the stage, entries with i < k ignored,
 * INT32_MAX = +infinity.
 *
 * Parity pins (tests marked "not gpu"): brute-force enumeration of Eq. 2 for
 * K <= 8, closed forms, the linear-partition reduction, invariants and
 * metamorphic relations.  No printed numeric example exists in the paper.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_K 256
#define ORC_INF32 INT32_MAX
#define ORC_INF64 INT64_MAX

typedef struct {
    int64_t T_star;                      /* ORC_INF64 if no feasible plan            */
    int32_t t_max;                       /* winning candidate                        */
    int32_t num_stages;                  /* 0 if infeasible                          */
    int32_t n_evaluated;                 /* candidates processed before the break    */
    int32_t first_layer[ORC_MAX_K + 1];  /* stage p = layers [first[p], first[p+1])  */
    int32_t shape_idx[ORC_MAX_K];
} orc_plan_t;

static int cmp_i32(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

/* Ascending, duplicates removed, in place.  Returns the new length. */
int orc_sort_dedup(int32_t *v, int n)
{
    if (n <= 0) return 0;
    qsort(v, (size_t)n, sizeof(int32_t), cmp_i32);
    int m = 1;
    for (int j = 1; j < n; ++j)
        if (v[j] != v[m - 1]) v[m++] = v[j];
    return m;
}

/* Alg. 1 "SortedAndFilter": every finite table value (entries with i >= k, all s,
 * all shapes), ascending, distinct.  out must hold K*K*K*S values.  Returns count. */
int orc_all_candidates(const int32_t *table, int K, int S, int32_t *out)
{
    int n = 0;
    for (int s = 0; s < K; ++s)
        for (int k = 0; k < K; ++k)
            for (int i = k; i < K; ++i)
                for (int q = 0; q < S; ++q) {
                    int32_t t = table[(((size_t)s * K + k) * K + i) * S + q];
                    if (t != ORC_INF32) out[n++] = t;
                }
    return orc_sort_dedup(out, n);
}

/* Evenly spaced quantiles of an ascending distinct list.  Returns count written. */
int orc_quantiles(const int32_t *v, int n, int Q, int32_t *out)
{
    if (n <= Q || Q < 2) {
        for (int j = 0; j < n; ++j) out[j] = v[j];
        return n;
    }
    for (int j = 0; j < Q; ++j)
        out[j] = v[((int64_t)j * (n - 1)) / (Q - 1)];
    return Q;
}

#define FIDX(s, k, d) ((((size_t)(s)) * (size_t)(K + 2) + (size_t)(k)) * (size_t)(D + 1) + (size_t)(d))

/* Eq. 3 for one candidate c: fills F[s][k][d] (s = 0..Smax, k = 0..K+1 (1-based
 * layers, index 0 unused), d = 0..D) and the arg-min (last layer i, 1-based, and
 * shape q) of every cell; -1 where F is infinite. */
void orc_fill_F(const int32_t *table, int K, int D, int S, const int32_t *a,
                int32_t c, int Smax, int64_t *F, int32_t *Ai, int32_t *Aq)
{
    size_t total = (size_t)(Smax + 1) * (size_t)(K + 2) * (size_t)(D + 1);
    for (size_t x = 0; x < total; ++x) { F[x] = ORC_INF64; Ai[x] = -1; Aq[x] = -1; }
    F[FIDX(0, K + 1, 0)] = 0;
    for (int s = 1; s <= Smax; ++s)
        for (int k = K; k >= 1; --k)
            for (int d = 1; d <= D; ++d) {
                int64_t best = ORC_INF64;
                int32_t bi = -1, bq = -1;
                for (int i = k; i <= K; ++i)
                    for (int q = 0; q < S; ++q) {
                        if (a[q] > d) continue;
                        int32_t t = table[((((size_t)(s - 1)) * K + (k - 1)) * K + (i - 1)) * S + q];
                        if (t == ORC_INF32 || t > c) continue;
                        int64_t p = F[FIDX(s - 1, i + 1, d - a[q])];
                        if (p == ORC_INF64) continue;
                        int64_t v = (int64_t)t + p;
                        if (v < best) { best = v; bi = i; bq = q; }
                    }
                F[FIDX(s, k, d)] = best;
                Ai[FIDX(s, k, d)] = bi;
                Aq[FIDX(s, k, d)] = bq;
            }
}

typedef struct {
    int64_t *F;
    int32_t *Ai, *Aq;
} orc_ws_t;

static int ws_alloc(orc_ws_t *w, int K, int D, int Smax)
{
    size_t total = (size_t)(Smax + 1) * (size_t)(K + 2) * (size_t)(D + 1);
    w->F = (int64_t *)malloc(total * sizeof(int64_t));
    w->Ai = (int32_t *)malloc(total * sizeof(int32_t));
    w->Aq = (int32_t *)malloc(total * sizeof(int32_t));
    return (w->F && w->Ai && w->Aq) ? 0 : -1;
}

static void ws_free(orc_ws_t *w)
{
    free(w->F); free(w->Ai); free(w->Aq);
}

/* Eq. 4 for one candidate, after orc_fill_F: returns T*(c) (or INF) and the
 * smallest s attaining the minimum; writes the plan by walking the arg-mins. */
static int64_t finish_candidate(const orc_ws_t *w, int K, int D, int Smax, int B,
                                int32_t c, const int32_t *a, int32_t *out_s, orc_plan_t *plan)
{
    int64_t ftot = ORC_INF64;
    int sbest = 0;
    for (int s = 1; s <= Smax; ++s) {
        int64_t f = w->F[FIDX(s, 1, D)];
        if (f < ftot) { ftot = f; sbest = s; }
    }
    if (out_s) *out_s = sbest;
    if (ftot == ORC_INF64) return ORC_INF64;
    int64_t T = ftot + (int64_t)(B - 1) * (int64_t)c;
    if (plan) {
        plan->T_star = T;
        plan->t_max = c;
        plan->num_stages = sbest;
        int s = sbest, k = 1, d = D, p = 0;
        while (s > 0) {
            int32_t i = w->Ai[FIDX(s, k, d)], q = w->Aq[FIDX(s, k, d)];
            plan->first_layer[p] = k - 1;
            plan->shape_idx[p] = q;
            ++p;
            d -= a[q];
            k = i + 1;
            --s;
        }
        plan->first_layer[p] = K;   /* k == K + 1 and d == 0 here */
    }
    return T;
}

/* T*(c) and s_c for candidates cand[j0..j1) (no pruning): the inner body of the
 * Alg. 1 loop, usable from a thread-per-candidate driver since candidates are
 * independent.  out_T / out_s are indexed like cand.  Returns 0, or -1 on OOM. */
int orc_eval_candidates(const int32_t *table, int K, int N, int M, int B,
                        const int32_t *shapes_nm, int S,
                        const int32_t *cand, int j0, int j1,
                        int64_t *out_T, int32_t *out_s)
{
    int D = N * M;
    int Smax = K < D ? K : D;
    int32_t a[64];
    if (S > 64 || K > ORC_MAX_K) return -2;
    for (int q = 0; q < S; ++q) a[q] = shapes_nm[2 * q] * shapes_nm[2 * q + 1];
    orc_ws_t w;
    if (ws_alloc(&w, K, D, Smax)) { ws_free(&w); return -1; }
    for (int j = j0; j < j1; ++j) {
        orc_fill_F(table, K, D, S, a, cand[j], Smax, w.F, w.Ai, w.Aq);
        int32_t sb;
        out_T[j] = finish_candidate(&w, K, D, Smax, B, cand[j], a, &sb, NULL);
        if (out_s) out_s[j] = sb;
    }
    ws_free(&w);
    return 0;
}

/* Plan of a single candidate (for the thread-driven path). */
int orc_plan_for(const int32_t *table, int K, int N, int M, int B,
                 const int32_t *shapes_nm, int S, int32_t c, orc_plan_t *plan)
{
    int D = N * M;
    int Smax = K < D ? K : D;
    int32_t a[64];
    if (S > 64 || K > ORC_MAX_K) return -2;
    for (int q = 0; q < S; ++q) a[q] = shapes_nm[2 * q] * shapes_nm[2 * q + 1];
    orc_ws_t w;
    if (ws_alloc(&w, K, D, Smax)) { ws_free(&w); return -1; }
    memset(plan, 0, sizeof(*plan));
    plan->T_star = ORC_INF64;
    orc_fill_F(table, K, D, S, a, c, Smax, w.F, w.Ai, w.Aq);
    int32_t sb;
    int64_t T = finish_candidate(&w, K, D, Smax, B, c, a, &sb, plan);
    if (T == ORC_INF64) { plan->T_star = ORC_INF64; plan->num_stages = 0; plan->t_max = 0; }
    ws_free(&w);
    return 0;
}

/* The inter-op DP loop of Alg. 1.  cand must be ascending and distinct.
 * out_T[j] (may be NULL) receives T*(cand[j]) for processed candidates, INF for
 * the ones after the pruning break. */
int orc_solve(const int32_t *table, int K, int N, int M, int B,
              const int32_t *shapes_nm, int S,
              const int32_t *cand, int C, int prune,
              int64_t *out_T, orc_plan_t *plan)
{
    int D = N * M;
    int Smax = K < D ? K : D;
    int32_t a[64];
    if (S > 64 || K > ORC_MAX_K) return -2;
    for (int q = 0; q < S; ++q) a[q] = shapes_nm[2 * q] * shapes_nm[2 * q + 1];
    orc_ws_t w;
    if (ws_alloc(&w, K, D, Smax)) { ws_free(&w); return -1; }
    orc_plan_t best, cur;
    memset(&best, 0, sizeof(best));
    best.T_star = ORC_INF64;
    if (out_T) for (int j = 0; j < C; ++j) out_T[j] = ORC_INF64;
    int processed = 0;
    for (int j = 0; j < C; ++j) {
        int32_t c = cand[j];
        if (prune && best.T_star != ORC_INF64 && (int64_t)B * (int64_t)c >= best.T_star) break;
        orc_fill_F(table, K, D, S, a, c, Smax, w.F, w.Ai, w.Aq);
        memset(&cur, 0, sizeof(cur));
        int64_t T = finish_candidate(&w, K, D, Smax, B, c, a, NULL, &cur);
        if (out_T) out_T[j] = T;
        ++processed;
        if (T < best.T_star) best = cur;
    }
    best.n_evaluated = processed;
    if (best.T_star == ORC_INF64) { best.num_stages = 0; best.t_max = 0; }
    *plan = best;
    ws_free(&w);
    return 0;
}

int orc_sizeof_plan(void) { return (int)sizeof(orc_plan_t); }
int orc_max_k(void) { return ORC_MAX_K; }
