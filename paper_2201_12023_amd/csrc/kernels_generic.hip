// General-size recurrence kernel (any K <= 256, N*M <= 1024), Eq. 4 / pruning / best
// selection, and plan recovery.  The recurrence here is the straightforward one: one
// workgroup per t_max candidate, threads over the cells (k, d) of a layer s, every cell
// scanning its (last layer, shape) terms in tie-break order; F layers live in global
// memory.  Problems of up to 128 layers on up to 128 devices normally run through the
// register/LDS kernel (fast_kernel.hpp); this one serves the remaining sizes.  Where that
// kernel does not recover the winner's layers itself (more than 64 devices), and for the
// remaining sizes, plan_layer_kernel does, one launch per layer.
#include "internal.hpp"

namespace alpa {

// F(s, k, d) of Eq. 3 for one candidate c, with F layers of (K+2) x (D+1) int32 each
// (k = 0..K+1, layers 1-based, k = K+1 is the "past the end" row; d = 0..D).
// layer(s) = slot + (s % n_layers) * layer_size.
// F(s, k, d) of Eq. 3 for candidate c from layer s-1 (`prev`), k and d 1-based; k_min: first
// layers below it are left at +infinity (the band of the plan-recovery run).
__device__ __forceinline__ int32_t relax_cell(const Problem &p, const int32_t *__restrict__ tab_s,
                                              const int32_t *__restrict__ sizes,
                                              const int32_t *__restrict__ prev, int32_t c, int s,
                                              int k, int d, int k_min)
{
    const int K = p.K, D = p.D, S = p.S;
    int32_t v = DEV_INF;
    // s stages need s layers and s devices: cells with k > K - s + 1 or d < s stay
    // infinite, and an operand F(s-1, i+1, .) can only be finite for K - i >= s - 1
    // (for s = 1 only the "past the end" row i + 1 = K + 1 is)
    if (k >= k_min && k <= K - s + 1 && d >= s) {
        const int i_first = (s == 1) ? K : k, i_last = K - s + 1;
        for (int i = i_first; i <= i_last; ++i) {
            const int32_t *tp = tab_s + ((size_t)(k - 1) * K + (i - 1)) * S;
            const int32_t *prow = prev + (i + 1) * (D + 1);
            for (int q = 0; q < S; ++q) {
                const int a = sizes[q];
                if (a > d) continue;
                const int32_t t = tp[q];
                if (t == INF_I32 || t > c) continue;
                const int32_t f = prow[d - a];
                if (f >= DEV_INF) continue;
                const int32_t sum = t + f;
                if (sum < v) v = sum;
            }
        }
    }
    return v;
}

__device__ void fill_layers(const Problem &p, const int32_t *__restrict__ table,
                            const int32_t *__restrict__ sizes, int32_t c, int32_t *slot,
                            int n_layers, int32_t *best_out, int32_t *sbest_out)
{
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    const int tid = threadIdx.x, nt = blockDim.x;
    // layer 0: only F(0, K+1, 0) = 0
    for (int x = tid; x < LS; x += nt) slot[x] = (x == (K + 1) * (D + 1)) ? 0 : DEV_INF;
    __syncthreads();
    int32_t best = DEV_INF, sbest = 0;
    for (int s = 1; s <= p.Smax; ++s) {
        const int32_t *prev = slot + (size_t)((s - 1) % n_layers) * LS;
        int32_t *cur = slot + (size_t)(s % n_layers) * LS;
        const int32_t *tab_s = table + (size_t)(s - 1) * K * K * S;
        for (int x = tid; x < LS; x += nt) {
            const int k = x / (D + 1), d = x - k * (D + 1);
            cur[x] = relax_cell(p, tab_s, sizes, prev, c, s, k, d, 1);
        }
        __syncthreads();
        const int32_t f1 = cur[1 * (D + 1) + D];       // F(s, first layer, all devices)
        if (f1 < best) { best = f1; sbest = s; }       // lowest s on ties
        __syncthreads();
    }
    *best_out = best;
    *sbest_out = sbest;
}

// In-flight use of the pruning rule (Alg. 1: stop once B * t_max >= best T*).  Candidate j
// may be skipped only on the evidence of finished candidates of LOWER index, because the
// sequential loop stops at the first index where the rule fires: the published running
// minima are kept per chunk of PRUNE_CHUNK candidates and only the chunks strictly below
// j's own are consulted.
__device__ bool can_skip(const int64_t *chunk_min, int j, int32_t c, int B)
{
    const int g = j / PRUNE_CHUNK;
    const int lane = threadIdx.x & (WAVE - 1);
    int64_t m = INF_I64;
    for (int x = lane; x < g; x += WAVE)
        m = min64(m, __atomic_load_n(&chunk_min[x], __ATOMIC_RELAXED));
    m = wave_min_i64(m);
    return m != INF_I64 && (int64_t)B * (int64_t)c >= m;
}

constexpr int GENERIC_MAX_THREADS = 1024;
__global__ __launch_bounds__(GENERIC_MAX_THREADS) void recurrence_generic_kernel(
    Problem p, const int32_t *__restrict__ table, const int32_t *__restrict__ sizes,
    const int32_t *__restrict__ cand, const int32_t *__restrict__ n_cand_p, int32_t *ticket,
    int64_t *chunk_min, int prune, int32_t *__restrict__ Fmin, int32_t *__restrict__ Sbest,
    int32_t *scratch, int n_layers)
{
    __shared__ int32_t sh_tk[GENERIC_MAX_THREADS];
    __shared__ int sh_skip[WAVE];
    const int LS = (p.K + 2) * (p.D + 1);
    int32_t *slot = scratch + (size_t)blockIdx.x * n_layers * LS;
    const int n = *n_cand_p;
    for (;;) {
        // No branch on the thread id in this loop (it would be loop-invariant and the
        // compiler may split the loop on it, letting lanes of a wave run out of step):
        // every thread issues the atomic, thread 0 adds 1 and the others 0, every thread
        // parks its return value and all read thread 0's.
        sh_tk[threadIdx.x] = atomicAdd(ticket, threadIdx.x == 0 ? 1 : 0);
        __syncthreads();
        const int j = sh_tk[0];
        __syncthreads();
        if (j >= n) break;                        // uniform exit: every wave reaches it
        const int32_t c = cand[j];
        if (prune) {
            const bool sk = can_skip(chunk_min, j, c, p.B);    // same value in every wave
            sh_skip[threadIdx.x & (WAVE - 1)] = sk ? 1 : 0;
            __syncthreads();
            const int skip = sh_skip[0];
            __syncthreads();
            if (skip) {
                Fmin[j] = DEV_INF;                // all threads, same value
                Sbest[j] = -1;
                continue;
            }
        }
        int32_t best, sbest;
        fill_layers(p, table, sizes, c, slot, n_layers, &best, &sbest);
        Fmin[j] = best;                           // all threads, same value
        Sbest[j] = best >= DEV_INF ? 0 : sbest;
        if (prune && best < DEV_INF)              // uniform; the minimum is idempotent
            atomicMin((long long *)&chunk_min[j / PRUNE_CHUNK],
                      (long long)best + (long long)(p.B - 1) * (long long)c);
        __syncthreads();
    }
}

// Plan recovery, one launch per layer: layer s (0..Smax) of the one candidate *c_p into
// F_all[s], every cell a thread, so that the whole device works on it (the single workgroup of
// recurrence_generic_kernel takes tens of milliseconds at the larger sizes).  Does nothing if
// *n_p == 0 (no winner) or s exceeds *s_top_p; only the cells the walk back from (s_top, first
// layer 1) can reach are computed.
__global__ __launch_bounds__(256) void plan_layer_kernel(
    Problem p, const int32_t *__restrict__ table, const int32_t *__restrict__ sizes,
    const int32_t *__restrict__ c_p, const int32_t *__restrict__ n_p,
    const int32_t *__restrict__ s_top_p, int s, int32_t *__restrict__ F_all)
{
    if (*n_p <= 0) return;
    const int s_top = min(p.Smax, *s_top_p);
    if (s > s_top) return;
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    int32_t *cur = F_all + (size_t)s * LS;
    if (s == 0) {                                  // only F(0, K+1, 0) = 0
        for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < LS; x += gridDim.x * blockDim.x)
            cur[x] = (x == (K + 1) * (D + 1)) ? 0 : DEV_INF;
        return;
    }
    const int32_t c = *c_p;
    const int32_t *prev = F_all + (size_t)(s - 1) * LS;
    const int32_t *tab_s = table + (size_t)(s - 1) * K * K * S;
    // a wave per cell, its lanes over the (last layer, shape) terms of the cell
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    const int k_min = max(1, s_top - s + 1);
    for (int x = wave; x < LS; x += n_waves) {
        const int k = x / (D + 1), d = x - k * (D + 1);
        int32_t v = DEV_INF;
        if (k >= k_min && k <= K - s + 1 && d >= s) {   // see relax_cell
            const int i_first = (s == 1) ? K : k, i_last = K - s + 1;
            const int n_terms = (i_last - i_first + 1) * S;
            const int32_t *tp = tab_s + ((size_t)(k - 1) * K + (i_first - 1)) * S;
            for (int j = lane; j < n_terms; j += WAVE) {
                const int di = j / S, q = j - di * S;
                const int a = sizes[q];
                if (a > d) continue;
                const int32_t t = tp[j];
                if (t == INF_I32 || t > c) continue;
                const int32_t f = prev[(i_first + di + 1) * (D + 1) + d - a];
                if (f >= DEV_INF) continue;
                v = min(v, t + f);
            }
        }
        for (int off = 32; off >= 1; off >>= 1) v = min(v, __shfl_xor(v, off, 64));
        if (lane == 0) cur[x] = v;
    }
}

// ---------------------------------------------------------------- Eq. 4 + best selection

// One block.  T(c_j) = Fmin_j + (B - 1) * c_j (Eq. 4); with pruning on, the processed set
// is the prefix [0, p) where p is the first index with B * c_p >= min_{j < p} T(c_j), as
// in the sequential loop of Alg. 1; the winner is the lowest T, lowest index on ties
// (strict "<" of Alg. 1 while ascending).
// `T` may be null (no per-candidate output).  One block of SEL_THREADS threads, tiles of
// SEL_THREADS candidates: prefix minimum inside each wave, the waves' totals through LDS, the
// first index that fires and the arg-min through LDS atomics.
constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / WAVE;

__device__ __forceinline__ void eq4_select(int B, int n, const int32_t *__restrict__ cand,
                                           const int32_t *__restrict__ Fmin,
                                           const int32_t *__restrict__ Sbest, SolveState *state,
                                           int prune, int64_t *__restrict__ T)
{
    __shared__ int64_t sh_wave_min[SEL_WAVES];
    __shared__ int sh_first_fire;
    __shared__ unsigned long long sh_best;             // lowest processed T of the tile
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid >> 6;
    int64_t carry = INF_I64;          // min of T over all earlier tiles
    int n_proc = n;
    int64_t bestT = INF_I64;
    int bestj = -1;
    bool stopped = false;             // block-uniform
    for (int j0 = 0; j0 < n; j0 += SEL_THREADS) {
        const int j = j0 + tid;
        if (stopped) {                // everything after the break is not evaluated
            if (T && j < n) T[j] = INF_I64;
            continue;
        }
        int64_t t = INF_I64, bc = 0;
        if (j < n) {
            const int32_t f = Fmin[j], c = cand[j];
            if (f < DEV_INF) t = (int64_t)f + (int64_t)(B - 1) * (int64_t)c;
            bc = (int64_t)B * (int64_t)c;
        }
        const int64_t incl = wave_prefix_min_i64(t, lane);
        if (tid == 0) { sh_first_fire = INT32_MAX; sh_best = ~0ull; }
        if (lane == WAVE - 1) sh_wave_min[w] = incl;
        __syncthreads();
        // exclusive prefix minimum: earlier tiles, earlier waves of this tile, earlier lanes
        int lo = __shfl_up(lo32(incl), 1, 64);
        int hi = __shfl_up(hi32(incl), 1, 64);
        int64_t excl = (lane == 0) ? INF_I64 : i64_from(lo, hi);
        excl = min64(excl, carry);
        int64_t tile_min = INF_I64;
        for (int x = 0; x < SEL_WAVES; ++x) {
            const int64_t m = sh_wave_min[x];
            if (x < w) excl = min64(excl, m);
            tile_min = min64(tile_min, m);
        }
        const bool fire = prune && j < n && excl != INF_I64 && bc >= excl;
        if (fire) atomicMin(&sh_first_fire, j);
        __syncthreads();
        const int first = sh_first_fire;               // INT32_MAX if nobody fired
        const bool processed = j < n && j < first;
        if (T && j < n) T[j] = processed ? t : INF_I64;
        // arg-min of the processed part of the tile in two steps: the lowest value (T >= 0, so
        // it orders as unsigned), then the lowest index that has it
        const int64_t tt = processed ? t : INF_I64;
        const int64_t wm = wave_min_i64(tt);
        if (lane == 0 && wm != INF_I64) atomicMin(&sh_best, (unsigned long long)wm);
        __syncthreads();
        const int64_t m = (int64_t)sh_best;            // ~0ull (= -1) if nothing finite
        __syncthreads();
        if (sh_best != ~0ull && m < bestT) {           // block-uniform
            if (tid == 0) sh_first_fire = INT32_MAX;   // reused: lowest index with T == m
            __syncthreads();
            if (tt == m) atomicMin(&sh_first_fire, j);
            __syncthreads();
            bestT = m;
            bestj = sh_first_fire;
        }
        __syncthreads();
        if (first != INT32_MAX) {
            n_proc = first;
            stopped = true;
        }
        carry = min64(carry, tile_min);
    }
    if (tid == 0) {
        state->n_processed = n_proc;
        state->best_idx = bestj;
        state->best_T = bestT;
        state->best_c = bestj >= 0 ? cand[bestj] : 0;
        state->best_s = bestj >= 0 ? Sbest[bestj] : 0;
        state->plan_n = bestj >= 0 ? 1 : 0;
        state->plan_ticket = 0;
    }
}

__global__ __launch_bounds__(SEL_THREADS) void epilogue_kernel(Problem p, const int32_t *__restrict__ cand,
                                                        const int32_t *__restrict__ Fmin,
                                                        const int32_t *__restrict__ Sbest,
                                                        SolveState *state, int prune,
                                                        int64_t *__restrict__ T)
{
    eq4_select(p.B, state->n_cand, cand, Fmin, Sbest, state, prune, T);
}

// Sweep over the number of microbatches: F of Eq. 3 does not depend on B, so one wave per
// B value applies Eq. 4 and the selection to the same Fmin / Sbest.  states[b] receives the
// winner for B_vals[b]; win_c / win_s are the compact copies the plan-recovery run reads.
__global__ __launch_bounds__(SEL_THREADS) void sweep_epilogue_kernel(
    const int32_t *__restrict__ B_vals, const int32_t *__restrict__ n_cand_p,
    const int32_t *__restrict__ cand, const int32_t *__restrict__ Fmin,
    const int32_t *__restrict__ Sbest, SolveState *states, int prune, int32_t *__restrict__ win_c,
    int32_t *__restrict__ win_s)
{
    const int b = blockIdx.x;
    SolveState *st = states + b;
    eq4_select(B_vals[b], *n_cand_p, cand, Fmin, Sbest, st, prune, nullptr);
    __syncthreads();                                   // lane 0's stores, then every lane's reads
    win_c[b] = st->best_c;                             // all lanes, same value
    win_s[b] = st->best_s;
}

// out_T in the caller's order: out_T[j] = T[rank_of_orig[j]]
__global__ void scatter_T_kernel(const int64_t *__restrict__ T, const int32_t *__restrict__ rank,
                                 int n_orig, int64_t *__restrict__ out_T)
{
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n_orig; j += gridDim.x * blockDim.x) {
        const int r = rank[j];
        out_T[j] = r >= 0 ? T[r] : INF_I64;
    }
}

__global__ void copy_T_kernel(const int64_t *__restrict__ T, const SolveState *state, int cap,
                              int64_t *__restrict__ out_T)
{
    int n = state->n_cand;
    if (n > cap) n = cap;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x)
        out_T[j] = T[j];
}

// ---------------------------------------------------------------- plan recovery

struct PlanDev {                       // same layout as alpa_plan_t (2072 bytes)
    int64_t T_star;
    int32_t t_max, num_stages, n_evaluated;
    int32_t first_layer[256 + 1];
    int32_t shape_idx[256];
};
static_assert(sizeof(PlanDev) == 2072, "PlanDev layout");

// One wave walks from (s*, first layer, all devices): at every step the (last layer, shape)
// terms are scanned in tie-break order, 64 at a time, and the first one that reproduces the
// stored F is taken (ballot + find-first-set = the wave-level arg-min with a fixed order).
__global__ __launch_bounds__(WAVE) void plan_walk_kernel(Problem p, const int32_t *__restrict__ table,
                                                         const int32_t *__restrict__ sizes,
                                                         const SolveState *state,
                                                         const int32_t *__restrict__ F_all,
                                                         size_t slab, PlanDev *plan,
                                                         PlanDev *best_plan)
{
    // block b recovers the plan of states[b] from the layers at F_all + b * slab
    __shared__ PlanDev sh;
    const int lane = threadIdx.x;
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    state += blockIdx.x;
    F_all += blockIdx.x * slab;
    plan += blockIdx.x;
    const bool feasible = state->best_idx >= 0;
    const int32_t c = state->best_c;
    const int64_t T_new = state->best_T;
    {
        const int n32 = (int)(sizeof(PlanDev) / 4);
        for (int x = lane; x < n32; x += WAVE) ((int32_t *)&sh)[x] = 0;
    }
    __syncthreads();
    int s = feasible ? state->best_s : 0;
    int k = 1, d = D, stage = 0;
    bool ok = true;
    while (s > 0) {
        const int32_t want = F_all[(size_t)s * LS + k * (D + 1) + d];
        const int n_terms = (K - k + 1) * S;
        int found = -1;
        for (int x0 = 0; x0 < n_terms && found < 0; x0 += WAVE) {
            const int x = x0 + lane;
            bool hit = false;
            if (x < n_terms) {
                const int i = k + x / S, q = x % S;
                const int a = sizes[q];
                if (a <= d) {
                    const int32_t t = table[(((size_t)(s - 1) * K + (k - 1)) * K + (i - 1)) * S + q];
                    if (t != INF_I32 && t <= c) {
                        const int32_t f = F_all[(size_t)(s - 1) * LS + (i + 1) * (D + 1) + (d - a)];
                        hit = f < DEV_INF && t + f == want;
                    }
                }
            }
            const uint64_t hm = __ballot(hit);
            if (hm) found = x0 + __ffsll((unsigned long long)hm) - 1;
        }
        if (found < 0 || want >= DEV_INF) { ok = false; break; }   // cannot happen for a consistent F
        const int i = k + found / S, q = found % S;
        sh.first_layer[stage] = k - 1;                 // all lanes, same value
        sh.shape_idx[stage] = q;
        ++stage;
        d -= sizes[q];
        k = i + 1;
        --s;
    }
    const bool good = feasible && ok;
    if (lane == 0) {
        if (good) sh.first_layer[stage] = K;
        sh.T_star = good ? T_new : INF_I64;
        sh.t_max = good ? c : 0;
        sh.num_stages = good ? stage : (feasible ? -1 : 0);   // -1 flags an internal inconsistency
        sh.n_evaluated = state->n_processed;
    }
    __syncthreads();
    // running best over all solves of the handle (not kept by sweeps: best_plan is null):
    // lower T*, then lower t_max
    const int64_t bT = best_plan ? best_plan->T_star : INF_I64;
    const int32_t bc = best_plan ? best_plan->t_max : 0;
    const bool better = best_plan && good && (T_new < bT || (T_new == bT && c < bc));
    const int n32 = (int)(sizeof(PlanDev) / 4);
    __syncthreads();
    for (int x = lane; x < n32; x += WAVE) {
        const int32_t v = ((const int32_t *)&sh)[x];
        ((int32_t *)plan)[x] = v;
        if (better) ((int32_t *)best_plan)[x] = v;
    }
}

__global__ void copy_plan_kernel(const PlanDev *src, PlanDev *dst)
{
    const int n32 = (int)(sizeof(PlanDev) / 4);
    for (int x = threadIdx.x; x < n32; x += blockDim.x)
        ((int32_t *)dst)[x] = ((const int32_t *)src)[x];
}

__global__ void init_state_kernel(SolveState *state, int64_t *chunk_min, int n_chunks)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) {
        state->ticket = 0;
        state->n_processed = 0;
        state->best_idx = -1;
        state->best_T = INF_I64;
        state->best_c = 0;
        state->best_s = 0;
        state->wave_relax = 0ull;
        state->plan_n = 0;
        state->plan_ticket = 0;
    }
    for (int x = t; x < n_chunks; x += gridDim.x * blockDim.x) chunk_min[x] = INF_I64;
}

__global__ void init_best_plan_kernel(PlanDev *best)
{
    const int n32 = (int)(sizeof(PlanDev) / 4);
    for (int x = threadIdx.x; x < n32; x += blockDim.x) ((int32_t *)best)[x] = 0;
    __syncthreads();
    if (threadIdx.x == 0) best->T_star = INF_I64;
}

// ---------------------------------------------------------------- launchers

hipError_t launch_recurrence_generic(hipStream_t st, const Problem &p, const int32_t *table,
                                     const int32_t *sizes, const int32_t *cand,
                                     const int32_t *n_cand_p, int32_t *ticket, int64_t *chunk_min,
                                     int prune, int32_t *Fmin, int32_t *Sbest, int32_t *scratch,
                                     int n_layers, int grid)
{
    // a lone workgroup (a single candidate) gets the widest block
    const int threads = grid == 1 ? GENERIC_MAX_THREADS : 256;
    hipLaunchKernelGGL(recurrence_generic_kernel, dim3(grid), dim3(threads), 0, st, p, table, sizes,
                       cand, n_cand_p, ticket, chunk_min, prune, Fmin, Sbest, scratch, n_layers);
    return hipGetLastError();
}

hipError_t launch_plan_layers(hipStream_t st, const Problem &p, const int32_t *table,
                              const int32_t *sizes, const int32_t *c_p, const int32_t *n_p,
                              const int32_t *s_top_p, int32_t *F_all)
{
    const int LS = (p.K + 2) * (p.D + 1);
    const int grid = std::min((LS + 3) / 4, 4096);     // four cells (waves) per block
    for (int s = 0; s <= p.Smax; ++s)
        hipLaunchKernelGGL(plan_layer_kernel, dim3(grid), dim3(256), 0, st, p, table, sizes, c_p,
                           n_p, s_top_p, s, F_all);
    return hipGetLastError();
}

hipError_t launch_epilogue(hipStream_t st, const Problem &p, const int32_t *cand,
                           const int32_t *Fmin, const int32_t *Sbest, SolveState *state, int prune,
                           int64_t *T)
{
    hipLaunchKernelGGL(epilogue_kernel, dim3(1), dim3(SEL_THREADS), 0, st, p, cand, Fmin, Sbest,
                       state, prune, T);
    return hipGetLastError();
}

hipError_t launch_scatter_T(hipStream_t st, const int64_t *T, const int32_t *rank_of_orig,
                            int n_orig, const SolveState *state, int64_t *out_T)
{
    int grid = (n_orig + 255) / 256;
    if (grid > 1024) grid = 1024;
    if (grid < 1) grid = 1;
    if (rank_of_orig)
        hipLaunchKernelGGL(scatter_T_kernel, dim3(grid), dim3(256), 0, st, T, rank_of_orig, n_orig,
                           out_T);
    else
        hipLaunchKernelGGL(copy_T_kernel, dim3(grid), dim3(256), 0, st, T, state, n_orig, out_T);
    return hipGetLastError();
}

hipError_t launch_plan_walk(hipStream_t st, const Problem &p, const int32_t *table,
                            const int32_t *sizes, SolveState *state, const int32_t *F_all,
                            void *plan_tmp, void *best_plan, void *plan_out)
{
    hipLaunchKernelGGL(plan_walk_kernel, dim3(1), dim3(WAVE), 0, st, p, table, sizes, state, F_all,
                       (size_t)0, (PlanDev *)plan_tmp, (PlanDev *)best_plan);
    if (plan_out && plan_out != plan_tmp)
        hipLaunchKernelGGL(copy_plan_kernel, dim3(1), dim3(256), 0, st, (const PlanDev *)plan_tmp,
                           (PlanDev *)plan_out);
    return hipGetLastError();
}

hipError_t launch_sweep_epilogue(hipStream_t st, const int32_t *B_vals, int n_B,
                                 const int32_t *n_cand_p, const int32_t *cand,
                                 const int32_t *Fmin, const int32_t *Sbest, SolveState *states,
                                 int prune, int32_t *win_c, int32_t *win_s)
{
    hipLaunchKernelGGL(sweep_epilogue_kernel, dim3(n_B), dim3(SEL_THREADS), 0, st, B_vals,
                       n_cand_p, cand, Fmin, Sbest, states, prune, win_c, win_s);
    return hipGetLastError();
}

hipError_t launch_plan_walk_many(hipStream_t st, const Problem &p, const int32_t *table,
                                 const int32_t *sizes, SolveState *states, const int32_t *F_all,
                                 size_t slab, void *plans, int n)
{
    hipLaunchKernelGGL(plan_walk_kernel, dim3(n), dim3(WAVE), 0, st, p, table, sizes, states, F_all,
                       slab, (PlanDev *)plans, (PlanDev *)nullptr);
    return hipGetLastError();
}

hipError_t launch_init_state(hipStream_t st, SolveState *state, int64_t *chunk_min, int n_chunks)
{
    int grid = (n_chunks + 255) / 256;
    if (grid < 1) grid = 1;
    if (grid > 256) grid = 256;
    hipLaunchKernelGGL(init_state_kernel, dim3(grid), dim3(256), 0, st, state, chunk_min, n_chunks);
    return hipGetLastError();
}

hipError_t launch_init_best_plan(hipStream_t st, void *best_plan)
{
    hipLaunchKernelGGL(init_best_plan_kernel, dim3(1), dim3(256), 0, st, (PlanDev *)best_plan);
    return hipGetLastError();
}

}  // namespace alpa
