// Register/LDS recurrence kernel (Eq. 3) for K <= 128 layers on N*M <= 64 devices, and on up
// to 128 devices in a two-window form (see WIDE below).  A header: the instances for up to 64
// and for 65-128 layers are compiled in two translation units (kernels_fast.hip,
// kernels_fast_deep.hip).
//
// Mapping.  One workgroup evaluates one t_max candidate at a time (persistent workgroups
// draw candidates from a ticket counter).  Lane l of every wave owns device count
// d = l + 1.  The first layers k are cut into half-blocks of 8; a workgroup has NWK =
// ceil(K / 16) waves along that axis and wave w owns half-blocks w ("A") and 2*NWK-1-w
// ("B"): the triangular work (a column with last layer i only touches first layers <= i)
// is then the same for every wave.  The 16 accumulators F(s, k, .) of a wave live in VGPRs;
// with WI > 1 the submesh shapes q are dealt round-robin over WI wave groups and the
// partial minima are merged through LDS.  The previous layer F(s-1, ., .) lives in LDS, one
// row of 64 lanes per first layer.  For a fixed (last layer i, shape q) the operand
// F(s-1, i+1, d - a_q) is one lane-shifted LDS row read, reused for all first layers of the
// wave, and t_intra(k..i, q, s) is the same for all lanes: it is fetched with scalar loads
// and used as the scalar operand of the add, so a cell-update costs one v_add and one v_min
// (one and a half instructions where two neighbouring columns are folded into one
// three-operand minimum: the one-candidate and the two-window forms).
// The filter t_intra <= t_max is wave-uniform; it is resolved per half-block from its
// precomputed min / max (skip, take unfiltered, or select per entry on the scalar unit).
// Infinite entries need no filter: DEV_INF + anything >= DEV_INF and accumulators start at
// DEV_INF.  Column loads (scalars and the LDS row) are issued one batch of two columns ahead.
// What is decided per shape (is there work for this wave in this layer, how many columns per
// half-block) is computed for all shapes at once, lane q for shape q, once per layer.
//
// Table layout (built once per handle by repack_fast_kernel): for every (s-1, q, half-block hb)
// a row of NP = ceil(K / 2) pair records, one per pair of neighbouring columns (last layers 2j
// and 2j+1), of PAIR_INTS = 22 int32:
//   [0..7]   t_intra of first layers 8hb..8hb+7 for last layer 2j      (DEV_INF where the first
//   [8..15]  the same for last layer 2j+1                                layer is > the last or
//   [16,17]  min, max over the finite entries of [0..15]                 >= K, or the entry is
//   [18,19]  max over the finite entries of [0..7], of [8..15]           +infinity)
//   [20,21]  min over the finite entries of [0..7], of [8..15]
// (DEV_INF for a minimum or maximum over nothing).  A wave walks its two rows front to
// back, so its scalar loads stream through whole cache lines, and the folded form fetches a
// batch (both columns of a pair) with one 16-dword and one 4-dword load.  The array is padded
// by a few records so that the loads that run ahead may pass the last row's end.
#pragma once
#include "internal.hpp"

#include <type_traits>

namespace alpa {

typedef const __attribute__((address_space(4))) int32_t *cptr_t;   // scalar-load path

constexpr int PAIR_INTS = 22;
constexpr int fast_pairs_per_row(int K) { return (K + 1) / 2; }
constexpr int END_SHAPES = 12;         // shapes covered by the early-stop table (3 registers)
// Rows of an F layer in LDS beyond the KP first layers.  Three, not more: with 64 layers a
// workgroup then takes 17152 + 3104 bytes of LDS and eight of them fit a compute unit.
constexpr int FAST_ROWS_SLACK = 3;

// Early-stop table: 8 groups of GW columns per (shape, half-block); GW = 8 up to 64 layers.
constexpr int END_GROUPS = 8;
constexpr int end_group_cols(int KP) { return KP > 64 ? KP / 8 : 8; }

// One half-block's share of a column, loaded one step ahead of its use.
struct HalfColumn {
    int32_t t[8];              // t_intra for 8 first layers (scalar registers)
    int32_t mn, mx;            // the half-block's min / max over finite entries
};

// half-column of absolute column `col` from the row `row` of its (s, q, half-block)
__device__ __forceinline__ void load_half(HalfColumn &h, cptr_t row, int col)
{
    const cptr_t pr = row + (uint32_t)(col >> 1) * PAIR_INTS;
    const int odd = col & 1;
    h.mn = pr[20 + odd];
    h.mx = pr[18 + odd];
#pragma unroll
    for (int u = 0; u < 8; ++u) h.t[u] = pr[8 * odd + u];
}
// both half-columns of the pair record at `pr`: x.mn / y.mn receive the PAIR's minimum and
// maximum (what the folded update classifies a batch by), x.mx / y.mx the half-columns' maxima
__device__ __forceinline__ void load_pair(HalfColumn &x, HalfColumn &y, cptr_t pr)
{
#pragma unroll
    for (int u = 0; u < 8; ++u) x.t[u] = pr[u];
#pragma unroll
    for (int u = 0; u < 8; ++u) y.t[u] = pr[8 + u];
    x.mn = pr[16]; y.mn = pr[17];
    x.mx = pr[18]; y.mx = pr[19];
}

// Makes loaded values "used" here, so that the wait for them is placed before the next
// loads are issued (scalar loads return out of order: any later wait would also wait for
// the loads just issued).  The memory clobber keeps later loads below this point.
__device__ __forceinline__ void settle(const HalfColumn &h)
{
    asm volatile("" :: "s"(h.t[0]), "s"(h.t[1]), "s"(h.t[2]), "s"(h.t[3]), "s"(h.t[4]),
                       "s"(h.t[5]), "s"(h.t[6]), "s"(h.t[7]), "s"(h.mn), "s"(h.mx)
                 : "memory");
}
__device__ __forceinline__ void settle(const HalfColumn &h, int32_t f)
{
    asm volatile("" :: "s"(h.t[0]), "s"(h.t[1]), "s"(h.t[2]), "s"(h.t[3]), "s"(h.t[4]),
                       "s"(h.t[5]), "s"(h.t[6]), "s"(h.t[7]), "s"(h.mn), "s"(h.mx), "v"(f)
                 : "memory");
}
__device__ __forceinline__ void fence_loads() { asm volatile("" ::: "memory"); }

// acc[off + u] = min(acc[off + u], t[u] + G) for the eight first layers of a half-block: the
// eight sums first, then the eight minima.  A v_min issued right behind the v_add it depends
// on holds the wave up; with only four waves per SIMD that caps the vector unit at 78 % of its
// issue rate (measured with a register-only loop: pairs 0.78, sums-then-minima 1.08 of one
// instruction per four clocks), so the sums are pinned in eight registers of their own.
__device__ __forceinline__ void relax_update(int32_t *acc, int off, const int32_t (&t)[8], int32_t G)
{
    int32_t sum[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) sum[u] = t[u] + G;
    asm volatile("" : "+v"(sum[0]), "+v"(sum[1]), "+v"(sum[2]), "+v"(sum[3]), "+v"(sum[4]),
                      "+v"(sum[5]), "+v"(sum[6]), "+v"(sum[7]));
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[off + u] = min(acc[off + u], sum[u]);
}

// Eight first layers against one column, for the NC candidates of the workgroup (ascending:
// c[0] <= c[1] <= ...).  A half-block is skipped when none of its entries passes the largest
// candidate, taken unfiltered when every finite entry passes the smallest, else filtered on
// the scalar unit candidate by candidate, from the largest down (the filtered set only
// shrinks, so the filter is applied in place).
template <int NC, bool COUNT>
__device__ __forceinline__ void relax8(int32_t (*acc)[16], int off, int32_t (&t)[8], int32_t mn,
                                       int32_t mx, const int32_t (&G)[NC], const int32_t (&c)[NC],
                                       unsigned &n_blocks)
{
    if (mn <= c[NC - 1]) {                    // else nothing passes even the largest candidate
#pragma unroll
        for (int e = NC - 1; e >= 0; --e) {   // largest candidate first: the filter only shrinks
            if (mx > c[e]) {
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = (t[u] <= c[e]) ? t[u] : DEV_INF;
            }
            if (COUNT) n_blocks += 8;
            relax_update(acc[e], off, t, G[e]);
            // (the next candidate filters the same eight registers in place: the compiler puts
            // its selects between this candidate's sums and minima)
            if (e > 0) asm volatile("" ::: "memory");
        }
    }
}

// Two columns of one half-block in one go (single candidate): acc = min3(acc, tX + GX, tY + GY),
// three vector instructions for two cell-updates per row instead of four.  Worth it where the
// kernel is bound by vector issue, which the one-candidate instances are (seven waves per SIMD).
// R < 8: only the first R first layers of the half-block (the others have no entry in these
// columns: see the diagonal columns in the kernel).
template <int R = 8>
__device__ __forceinline__ void relax_update2(int32_t *acc, int off, const int32_t (&tX)[8], int32_t GX,
                                              const int32_t (&tY)[8], int32_t GY)
{
#pragma unroll
    for (int h = 0; h < R; h += 4) {               // four rows at a time: eight sums in flight
        constexpr int N4 = 4;
        int32_t sx[N4], sy[N4];
#pragma unroll
        for (int u = 0; u < N4; ++u)
            if (h + u < R) { sx[u] = tX[h + u] + GX; sy[u] = tY[h + u] + GY; }
        if (h + 4 <= R)
            asm volatile("" : "+v"(sx[0]), "+v"(sx[1]), "+v"(sx[2]), "+v"(sx[3]), "+v"(sy[0]),
                              "+v"(sy[1]), "+v"(sy[2]), "+v"(sy[3]));
        else
            asm volatile("" : "+v"(sx[0]), "+v"(sx[1]), "+v"(sy[0]), "+v"(sy[1]));
#pragma unroll
        for (int u = 0; u < N4; ++u)
            if (h + u < R) acc[off + h + u] = min(acc[off + h + u], min(sx[u], sy[u]));
    }
}

// NW = 2: the two windows of device counts of a mesh of 65..128 devices (one candidate, so one
// filter; each window has its own accumulators and operands).
template <bool COUNT, int R = 8, int NW = 1>
__device__ __forceinline__ void relax8x2(int32_t (*acc)[16], int off, int32_t (&tX)[8], int32_t mnXY,
                                         int32_t mxX, const int32_t (&GX)[NW], int32_t (&tY)[8],
                                         int32_t mxXY, int32_t mxY, const int32_t (&GY)[NW], int32_t c,
                                         unsigned &n_blocks)
{
    // One path: skipped if the pair has no entry for the candidate (its minimum mnXY is above
    // it), taken as it is if every entry passes (its maximum mxXY does), else each half-column
    // is filtered where its own maximum exceeds the candidate.  A half-column with nothing for
    // the candidate has its maximum above it too, so the filter turns it into all-infinite
    // entries, which the minimum ignores: no separate code for "only one of the two", whose
    // extra exits cost the common path several taken branches.
    static_assert(R == 2 || R == 4 || R == 6 || R == 8, "rows of a diagonal batch");
    if (mnXY <= c) {
        if (mxXY > c) {
            if (mxX > c) {
#pragma unroll
                for (int u = 0; u < R; ++u) tX[u] = (tX[u] <= c) ? tX[u] : DEV_INF;
            }
            if (mxY > c) {
#pragma unroll
                for (int u = 0; u < R; ++u) tY[u] = (tY[u] <= c) ? tY[u] : DEV_INF;
            }
        }
        if (COUNT) n_blocks += 2 * R * NW;         // rows; a pair counts as two half-columns
#pragma unroll
        for (int w = 0; w < NW; ++w) relax_update2<R>(acc[w], off, tX, GX[w], tY, GY[w]);
    }
}

// Small meshes (GROUPED): the wave's lanes are cut into groups of DP = 2^ceil(log2 D) <= 32
// lanes, group g works for candidate j0 + g on device counts 1..DP, and all groups share every
// scalar t_intra.  The scalar side filters against the largest candidate of the wave (c_hi, as
// for a single candidate); entries between the smallest (c_lo) and c_hi pass for some groups
// only and are then filtered lane by lane against the lane's own candidate.
__device__ __forceinline__ void relax_update_lanes(int32_t *acc, int off, const int32_t (&t)[8],
                                                   int32_t G, int32_t c_lane)
{
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int32_t sum = (t[u] <= c_lane) ? t[u] + G : DEV_INF;
        acc[off + u] = min(acc[off + u], sum);
    }
}

template <bool COUNT>
__device__ __forceinline__ void relax8g(int32_t *acc, int off, int32_t (&t)[8], int32_t mn, int32_t mx,
                                        int32_t G, int32_t c_lo, int32_t c_hi, int32_t c_lane,
                                        unsigned &n_blocks)
{
    if (mn <= c_hi) {
        if (COUNT) n_blocks += 8;
        if (mx <= c_lo) relax_update(acc, off, t, G);
        else relax_update_lanes(acc, off, t, G, c_lane);
    }
}

template <bool COUNT>
__device__ __forceinline__ void relax8x2g(int32_t *acc, int off, int32_t (&tX)[8], int32_t mnXY,
                                          int32_t GX, int32_t (&tY)[8], int32_t mxXY, int32_t GY,
                                          int32_t c_lo, int32_t c_hi, int32_t c_lane,
                                          unsigned &n_blocks)
{
    // mnXY / mxXY: minimum and maximum over the finite entries of the pair
    if (mnXY <= c_hi) {
        if (COUNT) n_blocks += 16;
        if (mxXY <= c_lo) {
            relax_update2(acc, off, tX, GX, tY, GY);
        } else {
            // an entry above the lane's candidate turns into +infinity for that lane
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int32_t sx = (tX[u] <= c_lane) ? tX[u] + GX : DEV_INF;
                const int32_t sy = (tY[u] <= c_lane) ? tY[u] + GY : DEV_INF;
                acc[off + u] = min(acc[off + u], min(sx, sy));
            }
        }
    }
}

// Two candidates in one pass.  Where every device count a shape can still serve at this layer
// lies in one window of 32 (d - 1 in [base, base + 32)), lanes 0..31 work for candidate 0 and
// lanes 32..63 for candidate 1, both on that window: the scalar t_intra values are the same
// for both, so one add + min per first layer serves the two of them.  GP is the packed operand
// (lane l: F(s-1, i+1, d - a_q) of candidate l / 32), accP the packed accumulators.  If every
// finite entry passes both candidates one update does it; otherwise each candidate gets its
// own filtered update with the other half's operand set to infinity.
template <bool COUNT>
__device__ __forceinline__ void relax8p(int32_t (&accP)[16], int off, int32_t (&t)[8], int32_t mn,
                                        int32_t mx, int32_t GP, const int32_t (&c)[2], bool half1,
                                        unsigned &n_blocks)
{
    if (mn <= c[1]) {                         // else nothing passes even the larger candidate
        const bool both = mx <= c[0];
        if (mx > c[1]) {
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = (t[u] <= c[1]) ? t[u] : DEV_INF;
        }
        const int32_t G1 = (both || half1) ? GP : DEV_INF;
        if (COUNT) n_blocks += 8;
        relax_update(accP, off, t, G1);
        if (!both) {
            asm volatile("" : "+s"(t[0]), "+s"(t[1]), "+s"(t[2]), "+s"(t[3]), "+s"(t[4]),
                              "+s"(t[5]), "+s"(t[6]), "+s"(t[7]), "+v"(accP[off + 0]),
                              "+v"(accP[off + 1]), "+v"(accP[off + 2]), "+v"(accP[off + 3]),
                              "+v"(accP[off + 4]), "+v"(accP[off + 5]), "+v"(accP[off + 6]),
                              "+v"(accP[off + 7]));
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = (t[u] <= c[0]) ? t[u] : DEV_INF;
            const int32_t G0 = half1 ? DEV_INF : GP;
            if (COUNT) n_blocks += 8;
            relax_update(accP, off, t, G0);
        }
    }
}

// Lower-index evidence for the pruning rule (see recurrence_generic_kernel).
__device__ __forceinline__ bool can_skip_fast(const int64_t *chunk_min, int j, int32_t c, int B,
                                              int lane)
{
    const int g = j / PRUNE_CHUNK;
    int64_t m = INF_I64;
    for (int x = lane; x < g; x += WAVE)
        m = min64(m, __atomic_load_n(&chunk_min[x], __ATOMIC_RELAXED));
    m = wave_min_i64(m);
    return m != INF_I64 && (int64_t)B * (int64_t)c >= m;
}

// NWK = waves along the first-layer axis (= ceil(K / 16)); WI = wave groups along the shape
// axis; NC = candidates evaluated together by one workgroup (they share every scalar load);
// DUMP = also store every layer to F_all (plan recovery, NC = 1); COUNT = tally executed
// half-blocks.  Fmin / Sbest have a spare slot at index dummy_idx for results nobody owns.
// WIDE (with NC = 2): meshes of 65..128 devices.  One candidate per workgroup; the two
// accumulator sets and the two LDS regions that otherwise belong to two candidates hold the
// device counts 1..64 and 65..128 of the one candidate ("windows" 0 and 1).
// GROUPED (with NC = 1): meshes of up to 32 devices, 64 / DP candidates per workgroup (see
// relax8g above).
template <int NWK, int WI, int NC, bool DUMP, bool COUNT, bool WIDE = false, bool GROUPED = false>
// (The batch instances of the one-candidate form are meant to run eight waves per SIMD, i.e.
// in 64 vector registers.  Asking for eight here makes the compiler cut the scalar registers
// to 80 as well and spill; asked for seven it stays within 64 of its own accord, which the
// build step checks from the compiler's resource remarks.)
__global__ __launch_bounds__(WAVE * NWK * WI)
__attribute__((amdgpu_waves_per_eu((NC == 1 && WI == 1 && !DUMP && !WIDE && !GROUPED) ? 7 : 4)))
void recurrence_fast_kernel(
    Problem p, const int32_t *__restrict__ recs_g, const int32_t *__restrict__ sizes_g,
    const int32_t *__restrict__ cand, const int32_t *__restrict__ n_cand_p, int32_t *ticket,
    unsigned long long *wave_relax, int64_t *chunk_min, int prune, int descending,
    int32_t *__restrict__ Fmin, int32_t *__restrict__ Sbest, int dummy_idx,
    int32_t *__restrict__ F_all, const int32_t *__restrict__ s_top_p,
    const int32_t *__restrict__ group_min, int group_dp)
{
    static_assert((WI & (WI - 1)) == 0, "wave groups along the shape axis: a power of two");
    static_assert(!DUMP || NC == 1, "layer dump is for a single candidate");
    static_assert(!WIDE || (NC == 2 && WI == 1 && !DUMP), "two windows use the two-candidate layout");
    static_assert(!GROUPED || (NC == 1 && WI == 1 && !DUMP && !WIDE), "lane groups: one-candidate form");
    constexpr int NCAND = WIDE ? 1 : NC;               // candidates per workgroup (not GROUPED)
    constexpr int NT = WAVE * NWK * WI;
    constexpr int KP = NWK * 16;
    // LDS rows per F layer.  Column i reads row i + 1 <= K - 1 (layers s >= 2) and the loads run
    // at most two columns ahead of the last one: rows up to K + 1, so KP + 2 rows would do.
    constexpr int ROWS = KP + FAST_ROWS_SLACK;
    extern __shared__ int32_t lds[];                   // Fprev [NC][ROWS][64] (+ Fnext if WI > 1)
    __shared__ int32_t sh_tk[NWK * WI];
    __shared__ int32_t sh_skip[NWK * WI];
    // stage counts the early-stop table spans: 64, or 128 for more than 64 layers on more
    // than 64 devices (stage counts never exceed either)
    constexpr int SW = (WIDE && NWK > 4) ? 2 * WAVE : WAVE;
    __shared__ int32_t sh_ends[NWK * WI * (END_SHAPES / 4) * SW];     // early-stop table
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wid % NWK, wi = wid / NWK;
    const int hbA = wk, hbB = 2 * NWK - 1 - wk;        // the wave's two half-blocks of 8 first layers
    const int rowA = 8 * hbA, rowB = 8 * hbB;
    const int K = p.K, D = p.D, S = p.S;
    const int LS = (K + 2) * (D + 1);
    // int32 per (s, q, half-block) row; the whole array stays below 2^31 int32 (128 layers, 64
    // shapes: 1.8e8), so positions in it are 32-bit and only the pointer sum is 64-bit
    const uint32_t ROW = (uint32_t)fast_pairs_per_row(p.K) * PAIR_INTS;
    constexpr int NHB_ALL = KP / 8;
    constexpr int GW = end_group_cols(KP);             // columns per early-stop group
    const cptr_t recs = (cptr_t)recs_g;
    const cptr_t sizes = (cptr_t)sizes_g;
    int32_t *Fprev = lds;
    int32_t *Fnext = lds + NC * ROWS * WAVE;
    // candidate packing (two candidates, one pass): lane l works for candidate l / 32 on
    // device count d - 1 = pk_base + l % 32
    constexpr bool PACK = NC == 2 && WI == 1 && !DUMP && !WIDE;
    // one candidate per workgroup (batch and plan runs): two columns folded into one
    // three-operand minimum per row
    constexpr bool FOLD = NC == 1 || WIDE;
    const int pk_base = max(0, D - 32);
    const int pk_dl = pk_base + (lane & 31);
    const int pk_cand_off = (lane >> 5) * ROWS * WAVE;
    const bool half1 = lane >= 32;
    const int32_t size_of_lane = sizes[min(lane, S - 1)];   // lane q holds a_q (S <= 64)
    const int n = __builtin_amdgcn_readfirstlane(*n_cand_p);
    // GROUPED: lane = grp * DP + gl, group grp works for candidate j0 + grp on d - 1 = gl
    // (DP: a power of two, D <= DP <= 64, chosen by the host)
    const int DP = GROUPED ? group_dp : WAVE;
    const int ncand = GROUPED ? WAVE / DP : NCAND;     // candidates per workgroup
    const int gl = GROUPED ? (lane & (DP - 1)) : lane;
    const int grp = GROUPED ? lane / DP : 0;
    const int n_groups = (n + ncand - 1) / ncand;
    unsigned long long n_blocks_total = 0;

    for (;;) {
        // Every thread issues the atomic (thread 0 adds 1, the others 0) and all read thread
        // 0's return value.  No branch on the thread id may appear in this loop: it would be
        // loop-invariant, the compiler splits the loop on it, and the lanes of one wave then
        // run the persistent loop out of step with each other.
        // (each wave parks its first lane's return value; wave 0's first lane is thread 0)
        sh_tk[wid] = __builtin_amdgcn_readfirstlane(atomicAdd(ticket, tid == 0 ? 1 : 0));
        __syncthreads();
        const int tk = __builtin_amdgcn_readfirstlane(sh_tk[0]);
        __syncthreads();
        if (tk >= n_groups) break;                     // the workgroup's only exit
        const int j0 = (descending ? (n_groups - 1 - tk) : tk) * ncand;
        int jj[NC];                                    // candidate indices (the last may repeat;
        int32_t c[NC], c_given[NC];                    //  both windows serve one candidate)
#pragma unroll
        for (int e = 0; e < NC; ++e) {
            jj[e] = WIDE ? j0 : min(j0 + e, n - 1);
            c_given[e] = __builtin_amdgcn_readfirstlane(cand[jj[e]]);
            // as a filter every value from DEV_INF on is "no filter" (finite entries are far
            // below); clamped so that the sentinel entries themselves never pass it
            c[e] = min(c_given[e], DEV_INF - 1);
        }
        // GROUPED: every lane has its group's candidate; the scalar side works with the largest
        const int jl = min(j0 + grp, n - 1);
        int32_t c_lane_given = 0, c_lane = 0, c_lo = 0;
        if constexpr (GROUPED) {
            c_lane_given = cand[jl];
            c_lane = min(c_lane_given, DEV_INF - 1);
            c_lo = __builtin_amdgcn_readlane(c_lane, 0);         // candidates ascend with the group
            c[0] = __builtin_amdgcn_readlane(c_lane, WAVE - 1);
            c_given[0] = __builtin_amdgcn_readlane(c_lane_given, 0);   // decides the skip below
        }
        if (prune) {
            // If the lowest candidate of the group may be skipped so may the others (their
            // evidence set is a superset and B * t_max is larger).  Wave 0's reading of the
            // published minima decides for the whole workgroup.
            sh_skip[wid] = can_skip_fast(chunk_min, jj[0], c_given[0], p.B, lane) ? 1 : 0;
            __syncthreads();
            const int skip = __builtin_amdgcn_readfirstlane(sh_skip[0]);
            __syncthreads();
            if (skip) {
                if constexpr (GROUPED) {
                    Fmin[jl] = DEV_INF;                // every lane for its group's candidate
                    Sbest[jl] = -1;
                } else {
#pragma unroll
                    for (int e = 0; e < NCAND; ++e) {
                        Fmin[jj[e]] = DEV_INF;         // all threads, same value
                        Sbest[jj[e]] = -1;
                    }
                }
                continue;
            }
        }
        // Plan recovery walks back from F(s*, first layer 1, all devices): only layers up to
        // s* are needed, and of layer s only first layers (0-based) >= s* - s, since each of
        // the s* - s stages in front takes at least one layer.
        const int s_top =
            DUMP ? min(p.Smax, __builtin_amdgcn_readfirstlane(s_top_p[jj[0]])) : p.Smax;
        int32_t *F_out = DUMP ? F_all + (size_t)jj[0] * (size_t)(p.Smax + 1) * LS : nullptr;
        if (DUMP) {
            const int total = (s_top + 1) * LS;
            for (int x = tid; x < total; x += NT) F_out[x] = (x == (K + 1) * (D + 1)) ? 0 : DEV_INF;
            __syncthreads();
        }
        // Where the column loops may stop: lane s - 1 gets, for every shape q and the wave's two
        // half-blocks, the number of leading 8-column groups in which the largest candidate
        // still finds an entry (4 bits each, shape q at bits 8 (q % 4) of word q / 4 of the
        // wave's rows in sh_ends; only the wave itself reads them, so no barrier is needed).
        // Shapes beyond END_SHAPES are not covered (their loops run to the end).
        {
            const int32_t cmax = c[NC - 1];
            constexpr int NHB = KP / 8;
#pragma nounroll
            for (int ls = lane; ls < SW; ls += WAVE) { // s - 1 served by this lane
            int32_t word = 0;
#pragma nounroll
            for (int q = 0; q < END_SHAPES; ++q) {     // rows of shapes >= S are never read
                if (q < S) {
                    const int32_t *gA = group_min + ((q * NHB + hbA) * END_GROUPS) * SW + ls;
                    const int32_t *gB = group_min + ((q * NHB + hbB) * END_GROUPS) * SW + ls;
                    int nA = 0, nB = 0;
#pragma unroll
                    for (int j = 0; j < END_GROUPS; ++j) {
                        nA += gA[j * SW] <= cmax ? 1 : 0;
                        nB += gB[j * SW] <= cmax ? 1 : 0;
                    }
                    word |= (nA | (nB << 4)) << (8 * (q & 3));
                }
                if ((q & 3) == 3) {                    // four shapes per word
                    sh_ends[(wid * (END_SHAPES / 4) + (q >> 2)) * SW + ls] = word;
                    word = 0;
                }
            }
            }
        }
        int32_t best[NC], sbest[NC];
#pragma unroll
        for (int e = 0; e < NC; ++e) { best[e] = DEV_INF; sbest[e] = 0; }
        unsigned n_blocks = 0;
        // A launch that finds the records outside the L2 of its XCD (a first solve, or other
        // kernels since the last one) pays for it: the workgroups of an XCD walk the records
        // nearly in step at first, so a miss of one is a miss of all (workload 4: 4.2 instead of
        // 3.3 ms).  During about the first ticket of every workgroup (decided from the ticket
        // itself, so that the persistent loop is not peeled on it) each wave therefore touches,
        // a layer ahead, the part of its rows that the next layer reads.  The loads land in one
        // register that is never read; it stays reserved until the wait at the end of the ticket
        // (tied from asm to asm, so it keeps its place unless it is spilled: the build step
        // refuses a recurrence kernel that spills, to scratch or to accumulation registers).
        constexpr bool WARM = FOLD;
        // (more than 64 layers: the records of one candidate no longer fit the L2, every ticket
        // streams them in, so every ticket touches ahead)
        const bool warm_l2 = WARM && (NWK > 4 || tk < (int)gridDim.x);
        int32_t pf_touch = 0;
        // One layer of Eq. 3.  The first layer has a form of its own (the only finite operand is
        // F(0, K+1, 0) = 0) and is a separate instance of this body, in front of the loop over
        // the others: inside one loop the two forms meet at every shape, and the accumulators
        // are copied from one register set to another and back there.
        auto layer = [&](const int s, auto FIRST_T) {
            constexpr bool FIRST = decltype(FIRST_T)::value;
            const bool needA = !DUMP || rowA + 7 >= s_top - s;
            const bool needB = !DUMP || rowB + 7 >= s_top - s;
            auto mnA = [&](const HalfColumn &h) { return needA ? h.mn : DEV_INF; };   // "no entry
            auto mnB = [&](const HalfColumn &h) { return needB ? h.mn : DEV_INF; };   //  passes"
            int32_t acc[NC][16];                       // [0..7] half-block A, [8..15] half-block B
#pragma unroll
            for (int e = 0; e < NC; ++e)
#pragma unroll
                for (int u = 0; u < 16; ++u) acc[e][u] = DEV_INF;
            int32_t accP[16];                          // packed passes (PACK only)
#pragma unroll
            for (int u = 0; u < 16; ++u) accP[u] = DEV_INF;
            int32_t c2[2] = {c[0], c[NC - 1]};
            if constexpr (WARM) {
                if (warm_l2 && s < s_top) {
                    // layer s + 1 has columns up to K - s - 1; 128 bytes a lane, lanes 0..31 for
                    // half-block A's row and 32..63 for B's (rows of 64 layers have 2816 bytes)
                    // (more than 64 layers: rows of up to 5632 bytes, all 64 lanes for A's row
                    // and a second load for B's)
                    constexpr int LANES = NWK <= 4 ? 32 : WAVE;
                    const int hi = (((K - s - 1) >> 1) + 1) * PAIR_INTS - 1;
                    const int hb = (NWK <= 4 && (lane & 32)) ? hbB : hbA;
                    const int lo = 4 * hb * PAIR_INTS;                     // pair of column 8 hb
                    const int at = min(lo + 32 * (lane & (LANES - 1)), max(lo, hi));
                    const int32_t *row = recs_g + (((uint32_t)s * S * NHB_ALL + hb) * ROW + at);
                    const int loB = 4 * hbB * PAIR_INTS;
                    const int atB = min(loB + 32 * lane, max(loB, hi));
                    const int32_t *rowB2 = recs_g + (((uint32_t)s * S * NHB_ALL + hbB) * ROW + atB);
                    for (int q = wi; q < S; q += WI) {
                        const int a = __builtin_amdgcn_readlane(size_of_lane, q);
                        if (a + s > D) continue;               // the shape leaves no device to s stages
                        const int32_t *ptr = row + (uint32_t)q * NHB_ALL * ROW;
                        asm volatile("global_load_dword %0, %1, off" : "+v"(pf_touch) : "v"(ptr) : "memory");
                        if constexpr (NWK > 4) {
                            const int32_t *ptrB = rowB2 + (uint32_t)q * NHB_ALL * ROW;
                            asm volatile("global_load_dword %0, %1, off" : "+v"(pf_touch) : "v"(ptrB) : "memory");
                        }
                    }
                }
            }
            // the layer's early-stop counts, those of shape q in lane q (one LDS read per layer
            // instead of one per shape); shapes beyond the table get "all eight groups".  (A
            // select, not a branch on the lane id: see the ticket comment.)
            const int32_t ends_word =
                sh_ends[(wid * (END_SHAPES / 4) + min(lane >> 2, END_SHAPES / 4 - 1)) * SW + s - 1];
            const int32_t ends_of_lane = lane < END_SHAPES ? (ends_word >> (8 * (lane & 3))) & 0xff : 0x88;
            const int i_lo = FIRST ? K - 1 : 0;        // 0-based last layer
            const int i_hi = K - s;                    // at least s-1 layers must remain
            const int i0 = max(i_lo, rowA);            // columns that reach half-block A
            // Which shapes this wave has work for in this layer, decided for all of them at once
            // (lane q for shape q): the shape leaves a device to each of the s - 1 stages behind,
            // the wave has columns at all, and the largest candidate still finds an entry in
            // reach of one of its half-blocks.  The shape loop then walks the set bits.
            const int32_t endA_l = needA ? GW * (ends_of_lane & 15) : 0;
            const int32_t endB_l = needB ? GW * ((ends_of_lane >> 4) & 15) : 0;
            const bool alive_l = lane < S && (lane & (WI - 1)) == wi && size_of_lane + s - 1 <= D &&
                                 i0 <= i_hi && (FIRST || !(endA_l <= i0 && endB_l <= rowB));
            // packed (two-candidate form) when every device count the shape can still serve is
            // in the window
            const bool packed_l = PACK && !FIRST && size_of_lane + s - 2 >= pk_base;
            // folded form: the column counts of the two half-block passes, A's in bits 0..7 and
            // B's in bits 8..15
            const int cB0 = max(i0, rowB);
            const int32_t counts_l = max(0, min(i_hi + 1, endA_l) - i0) |
                                     (max(0, min(i_hi + 1, endB_l) - cB0) << 8);
            if (WI > 1) {
                for (int x = tid; x < NC * ROWS * WAVE; x += NT) Fnext[x] = DEV_INF;
            }
            bool packed_any = false;                   // a packed pass touched accP
            // Two passes over the shapes: first those whose updates go candidate by candidate,
            // then those served by the packed form (one pass at a time keeps each loop's set
            // of live accumulators, and with it the register traffic between them, small).
            auto shapes_pass = [&](auto PASS_PACKED) {
            constexpr bool PASS_P = decltype(PASS_PACKED)::value;
            // (wave group wi takes every WI-th shape)
            unsigned long long todo = __ballot(alive_l && packed_l == PASS_P);
            while (todo) {
                const int q = __builtin_ctzll(todo);
                todo &= todo - 1;
                const int a = __builtin_amdgcn_readlane(size_of_lane, q);
                // first column group without anything for the largest candidate, per half-block
                // (the folded form takes its column counts from counts_l instead)
                int endA = 0, endB = 0;
                if constexpr (!FOLD) {
                    const int bits = __builtin_amdgcn_readlane(ends_of_lane, q);
                    endA = needA ? GW * (bits & 15) : 0;
                    endB = needB ? GW * ((bits >> 4) & 15) : 0;
                }
                if (PASS_P) packed_any = true;
                const uint32_t rowsq = ((uint32_t)(s - 1) * S + q) * NHB_ALL * ROW;
                const cptr_t pA = recs + (rowsq + hbA * ROW);                   // the wave's two rows
                const cptr_t pB = recs + (rowsq + hbB * ROW);
                const int ncol = i_hi - i0 + 1;                // columns of this wave
                HalfColumn hA, hB;
                int32_t G[NC];
                if constexpr (FIRST) {
                    // F(0, K+1, 0) = 0 is the only finite operand: last layer K-1, d = a_q
#pragma unroll
                    for (int e = 0; e < NC; ++e)
                        G[e] = ((WIDE ? WAVE * e : 0) + gl + 1 == a) ? 0 : DEV_INF;
                    int i = i0;
                    for (int x = 0; x < ncol; ++x, ++i) {
                        load_half(hA, pA, i);
                        load_half(hB, pB, i);
                        if constexpr (GROUPED) {
                            relax8g<COUNT>(acc[0], 0, hA.t, hA.mn, hA.mx, G[0], c_lo, c[0], c_lane, n_blocks);
                            if (i >= rowB)
                                relax8g<COUNT>(acc[0], 8, hB.t, hB.mn, hB.mx, G[0], c_lo, c[0], c_lane, n_blocks);
                        } else {
                            relax8<NC, COUNT>(acc, 0, hA.t, mnA(hA), hA.mx, G, c, n_blocks);
                            if (i >= rowB) relax8<NC, COUNT>(acc, 8, hB.t, mnB(hB), hB.mx, G, c, n_blocks);
                        }
                    }
                } else {
                auto columns = [&](auto PK) {
                    // Pipeline, one batch ahead.  A batch is two half-columns (slots X and Y) with
                    // their LDS rows; while one batch is computed the loads of the next are in
                    // flight, so every wait is covered by a whole batch of updates.  Three
                    // phases: columns that reach only half-block A (a batch = the A halves of two
                    // columns), columns in which both half-blocks still have entries for the
                    // largest candidate (a batch = the A and B halves of one column), and the
                    // columns in which only half-block B has (a batch = the B halves of two
                    // columns).  Loads past the last column land in the padding and are dropped.
                    // P: the two candidates share each pass (see relax8p); one LDS row per column
                    constexpr bool P = decltype(PK)::value;
                    constexpr int NF = P ? 1 : NC;
                    const int dl = P ? pk_dl : lane;       // d - 1 served by this lane
                    const bool live = (GROUPED ? gl : dl) >= a;   // d - a_q >= 1
                    // window 1 (WIDE): d - 1 = 64 + lane; its operand d - a_q lies in window 1
                    // for lane >= a_q, else in window 0 at lane 64 + lane - a_q
                    const bool live1 = WAVE + lane >= a;
                    const int wide_delta = (lane >= a ? ROWS * WAVE + lane - a
                                                      : max(0, WAVE + lane - a)) -
                                           (live ? lane - a : 0);
                    auto row_ptr = [&](int i) {            // operand row of column i: row i + 1
                        return Fprev + (P ? pk_cand_off : 0) + (live ? dl - a : 0) + (i + 1) * WAVE;
                    };
                    struct Batch { HalfColumn X, Y; int32_t fX[NF], fY[NF]; } b0, b1;
                    auto operands = [&](const int32_t (&src)[NF]) {
#pragma unroll
                        for (int e = 0; e < NF; ++e)
                            G[e] = ((WIDE && e == 1) ? live1 : live) ? src[e] : DEV_INF;
                    };
                    auto relax = [&](int off, HalfColumn &h, int32_t mn) {
                        if constexpr (P)
                            relax8p<COUNT>(accP, off, h.t, mn, h.mx, G[0], c2, half1, n_blocks);
                        else if constexpr (GROUPED)
                            relax8g<COUNT>(acc[0], off, h.t, mn, h.mx, G[0], c_lo, c[0], c_lane, n_blocks);
                        else
                            relax8<NC, COUNT>(acc, off, h.t, mn, h.mx, G, c, n_blocks);
                    };
                    // `count` columns from column c0 (frow: its operand row) of the row `row`,
                    // one half-block (acc rows off..off+7) only; folded: c0 is even
                    auto single = [&](int off, cptr_t row, int c0, const int32_t *frow, int count, auto mnf) {
                        cptr_t pp = row + (uint32_t)(c0 >> 1) * PAIR_INTS; // folded: pair of column c0
                        auto rows = [&](int32_t (&dst)[NF], int col) {
#pragma unroll
                            for (int e = 0; e < NF; ++e)
                                dst[e] = frow[(WIDE && e == 1 ? wide_delta : e * ROWS * WAVE) + col * WAVE];
                        };
                        auto load2 = [&](Batch &b, int col) {
                            rows(b.fX, col);
                            rows(b.fY, col + 1);
                            if constexpr (FOLD) {
                                load_pair(b.X, b.Y, pp + (col >> 1) * PAIR_INTS);
                            } else {
                                load_half(b.X, row, c0 + col);
                                load_half(b.Y, row, c0 + col + 1);
                            }
                            fence_loads();
                        };
                        // the first eight columns of a half-block's own pass are its diagonal:
                        // column 8hb + j has entries for the first layers 8hb .. 8hb + j only, so
                        // the batch of columns j = 2b, 2b+1 needs the first 2b + 2 rows
                        // folded form: the operands as they come (only the lanes that have one
                        // are switched on); with two windows the lanes below the shape's size
                        // have one in window 1 only
                        auto fold_operands = [&](Batch &b) {
                            if constexpr (WIDE) {
                                b.fX[0] = live ? b.fX[0] : DEV_INF;
                                b.fY[0] = live ? b.fY[0] : DEV_INF;
                            }
                        };
                        auto compute2_rows = [&](Batch &b, auto ROWS_T) {
                            fold_operands(b);
                            relax8x2<COUNT, decltype(ROWS_T)::value, NF>(acc, off, b.X.t, mnf(b.X), b.X.mx,
                                                                         b.fX, b.Y.t, b.Y.mn, b.Y.mx,
                                                                         b.fY, c[0], n_blocks);
                        };
                        auto compute2 = [&](Batch &b) {
                            if constexpr (GROUPED) {
                                relax8x2g<COUNT>(acc[0], off, b.X.t, mnf(b.X), b.fX[0], b.Y.t, b.Y.mn,
                                                 b.fY[0], c_lo, c[0], c_lane, n_blocks);
                            } else if constexpr (FOLD) {
                                fold_operands(b);
                                relax8x2<COUNT, 8, NF>(acc, off, b.X.t, mnf(b.X), b.X.mx, b.fX, b.Y.t,
                                                       b.Y.mn, b.Y.mx, b.fY, c[0], n_blocks);
                            } else {
                                operands(b.fX);
                                relax(off, b.X, mnf(b.X));
                                operands(b.fY);
                                relax(off, b.Y, mnf(b.Y));
                            }
                        };
                        auto settle2 = [&](const Batch &b) {
                            settle(b.X, b.fX[0]);
                            settle(b.Y, b.fY[0]);
                        };
                        int left = count;
                        if (left >= 2) {
                            load2(b0, 0);
                            if constexpr (FOLD && !GROUPED) {
                                if (left >= 8) {           // (c0 is the half-block's first column)
                                    settle2(b0);
                                    load2(b1, 2);
                                    compute2_rows(b0, std::integral_constant<int, 2>{});
                                    settle2(b1);
                                    load2(b0, 4);
                                    compute2_rows(b1, std::integral_constant<int, 4>{});
                                    settle2(b0);
                                    load2(b1, 6);
                                    compute2_rows(b0, std::integral_constant<int, 6>{});
                                    settle2(b1);
                                    load2(b0, 8);
                                    compute2(b1);
                                    pp += 4 * PAIR_INTS;
                                    c0 += 8;
                                    frow += 8 * WAVE;
                                    left -= 8;
                                }
                            }
                            if constexpr (FOLD && !GROUPED) {
                                for (; left >= 8; left -= 8) {   // (loop control once per four batches)
                                    settle2(b0);
                                    load2(b1, 2);
                                    compute2(b0);
                                    settle2(b1);
                                    load2(b0, 4);
                                    compute2(b1);
                                    settle2(b0);
                                    load2(b1, 6);
                                    compute2(b0);
                                    settle2(b1);
                                    load2(b0, 8);
                                    compute2(b1);
                                    pp += 4 * PAIR_INTS;
                                    c0 += 8;
                                    frow += 8 * WAVE;
                                }
                            }
                            for (; left >= 4; left -= 4) {
                                settle2(b0);
                                load2(b1, 2);
                                compute2(b0);
                                settle2(b1);
                                load2(b0, 4);
                                compute2(b1);
                                pp += 2 * PAIR_INTS;
                                c0 += 4;
                                frow += 4 * WAVE;
                            }
                            if (left >= 2) {
                                settle2(b0);
                                compute2(b0);
                                pp += PAIR_INTS;
                                c0 += 2;
                                frow += 2 * WAVE;
                                left -= 2;
                            }
                        }
                        if (left == 1) {
                            rows(b0.fX, 0);
                            load_half(b0.X, row, c0);
                            operands(b0.fX);
                            relax(off, b0.X, mnf(b0.X));
                        }
                    };
                    // columns of each phase; endA / endB bound where the half-blocks still
                    // have something for the largest candidate
                    if constexpr (FOLD) {
                        // every column pair of a half-block folds, so the half-blocks go one
                        // after the other (the operand row of a column is read once for each)
                        // Lanes below the shape's size have no operand (d - a_q < 1) and nothing
                        // to update: they sit the pass out, which saves the select of the
                        // operand per column.  (Not a branch on the lane id alone: the set
                        // changes with the shape, so the loops around are not split on it.)
                        const int counts = __builtin_amdgcn_readlane(counts_l, q);
                        if (WIDE ? live1 : live) {
                            single(0, pA, i0, row_ptr(i0), counts & 0xff, mnA);
                            single(8, pB, cB0, row_ptr(cB0), counts >> 8, mnB);
                        }
                        return;
                    }
                    const int n1 = max(0, min(rowB - i0, ncol));       // reach half-block A only
                    const int cAB = i0 + n1;                           // first column reaching B
                    const int stopAB = endA > endB ? endA : min(endA, endB);
                    const int nAB = max(0, min(ncol - n1, stopAB - cAB));
                    const int cB = cAB + nAB;                          // B alone from here
                    const int nB = max(0, min(i_hi + 1, endB) - cB);
                    single(0, pA, i0, row_ptr(i0), max(0, min(n1, endA - i0)), mnA);
                    {
                        int cc = cAB;                                  // column of the next batch
                        const int32_t *frow = row_ptr(cAB);
                        auto load_AB = [&](Batch &b, int col) {
#pragma unroll
                            for (int e = 0; e < NF; ++e)
                                b.fX[e] = frow[(WIDE && e == 1 ? wide_delta : e * ROWS * WAVE) + col * WAVE];
                            load_half(b.X, pA, cc + col);
                            load_half(b.Y, pB, cc + col);
                            fence_loads();
                        };
                        auto compute_AB = [&](Batch &b) {
                            operands(b.fX);
                            relax(0, b.X, mnA(b.X));
                            relax(8, b.Y, mnB(b.Y));
                        };
                        auto settle_AB = [&](const Batch &b) {
                            settle(b.X, b.fX[0]);
                            settle(b.Y);
                        };
                        int left = nAB;
                        if (left >= 1) {
                            load_AB(b0, 0);
                            for (; left >= 2; left -= 2) {
                                settle_AB(b0);
                                load_AB(b1, 1);
                                compute_AB(b0);
                                settle_AB(b1);
                                load_AB(b0, 2);
                                compute_AB(b1);
                                cc += 2;
                                frow += 2 * WAVE;
                            }
                            if (left == 1) {
                                settle_AB(b0);
                                compute_AB(b0);
                            }
                        }
                    }
                    single(8, pB, cB, row_ptr(cB), nB, mnB);
                };
                columns(PASS_PACKED);
                }
            }
            };
            shapes_pass(std::false_type{});
            if constexpr (PACK) shapes_pass(std::true_type{});
            if (PACK && packed_any) {
                // lane l (d - 1 = l) takes candidate e's packed result from lane 32 e + l - pk_base
                const int rel = lane - pk_base;
                const bool in_window = rel >= 0 && rel < 32;
#pragma unroll
                for (int e = 0; e < NC; ++e)
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int32_t v = __shfl(accP[u], (32 * e + rel) & 63, 64);
                        acc[e][u] = min(acc[e][u], in_window ? v : DEV_INF);
                    }
            }
            __syncthreads();                           // every wave is done reading Fprev
            int32_t f1[NC];
            if (WI == 1) {
#pragma unroll
                for (int e = 0; e < NC; ++e)
#pragma unroll
                    for (int u = 0; u < 8; ++u) {      // rows 0 and >= K are never operands
                        Fprev[(e * ROWS + rowA + u) * WAVE + lane] = acc[e][u];
                        Fprev[(e * ROWS + rowB + u) * WAVE + lane] = acc[e][8 + u];
                    }
                __syncthreads();
#pragma unroll
                for (int e = 0; e < NC; ++e) f1[e] = acc[e][0];   // F(s, first layer, .) in wave 0
            } else {
#pragma unroll
                for (int e = 0; e < NC; ++e)
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        atomicMin(&Fnext[(e * ROWS + rowA + u) * WAVE + lane], acc[e][u]);
                        atomicMin(&Fnext[(e * ROWS + rowB + u) * WAVE + lane], acc[e][8 + u]);
                    }
                __syncthreads();
                int32_t *tmp = Fprev; Fprev = Fnext; Fnext = tmp;
#pragma unroll
                for (int e = 0; e < NC; ++e) f1[e] = Fprev[e * ROWS * WAVE + lane];   // row 0
            }
#pragma unroll
            for (int e = 0; e < NC; ++e)
                if (f1[e] < best[e]) { best[e] = f1[e]; sbest[e] = s; }   // lowest s on ties
            if (DUMP) {
                int32_t *Fs = F_out + (size_t)s * LS;
                if (WI == 1) {
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int k = (u < 8 ? rowA : rowB - 8) + u;
                        const bool in = lane < D;
                        if (k < K) Fs[(k + 1) * (D + 1) + (in ? lane + 1 : 0)] = in ? acc[0][u] : DEV_INF;
                    }
                } else {
                    // lanes beyond the mesh rewrite the row's d = 0 cell with infinity
                    // (a select, not a branch on the lane id: see the ticket comment)
                    for (int x = tid; x < K * WAVE; x += NT) {
                        const int k = x >> 6, l = x & (WAVE - 1);
                        const bool in = l < D;
                        Fs[(k + 1) * (D + 1) + (in ? l + 1 : 0)] = in ? Fprev[x] : DEV_INF;
                    }
                }
            }
        };
        if (s_top >= 1) layer(1, std::true_type{});
        for (int s = 2; s <= s_top; ++s) layer(s, std::false_type{});
        if constexpr (WARM) asm volatile("s_waitcnt vmcnt(0)" : "+v"(pf_touch) :: "memory");
        if constexpr (GROUPED) {
            // the lane of device count D in group grp holds F(s, first layer, all devices) of
            // candidate j0 + grp; every other lane (and every wave but wave 0) stores to the
            // spare slot
            const bool owner = (wid == 0) && (gl == D - 1) && (j0 + grp < n);
            const int slot = owner ? jl : dummy_idx;
            Fmin[slot] = best[0];
            Sbest[slot] = best[0] >= DEV_INF ? 0 : sbest[0];
            // one atomic per candidate (the owner changes with the ticket: not a branch the
            // persistent loop could be split on)
            if (prune && owner && best[0] < DEV_INF)
                atomicMin((long long *)&chunk_min[jl / PRUNE_CHUNK],
                          (long long)best[0] + (long long)(p.B - 1) * (long long)c_lane_given);
        } else {
        // lane D-1 (of window (D-1)/64) holds F(s, first layer, all devices); wave 0 owns the
            // results; a repeated last candidate goes to the spare slot
#pragma unroll
            for (int e = 0; e < NCAND; ++e) {
                const int32_t bv = (WIDE && D > WAVE) ? best[NC - 1] : best[e];
                const int32_t sv = (WIDE && D > WAVE) ? sbest[NC - 1] : sbest[e];
                const int32_t bestD = __builtin_amdgcn_readlane(bv, (D - 1) & (WAVE - 1));
                const int32_t sD = __builtin_amdgcn_readlane(sv, (D - 1) & (WAVE - 1));
                const bool owner = (wid == 0) && (j0 + e < n);
                const int slot = owner ? jj[e] : dummy_idx;
                Fmin[slot] = bestD;                        // all lanes, same value
                Sbest[slot] = bestD >= DEV_INF ? 0 : sD;
                if (prune) {                               // uniform; the minimum is idempotent
                    const long long T = (owner && bestD < DEV_INF)
                                            ? (long long)bestD + (long long)(p.B - 1) * (long long)c_given[e]
                                            : (long long)INF_I64;
                    atomicMin((long long *)&chunk_min[jj[e] / PRUNE_CHUNK], T);
                }
            }
        }
        if (COUNT) n_blocks_total += n_blocks;
        __syncthreads();                               // LDS is reused by the next group
    }
    // (the last lane: it takes part in every pass, also where the low lanes sit one out)
    // n_blocks counts rows (64-lane add + minimum groups) of the updates executed
    if (COUNT) atomicAdd(wave_relax, lane == WAVE - 1 ? n_blocks_total : 0ull);
}

// shape-axis wave groups of the single-candidate (plan) run: as many as 1024 threads allow
constexpr int plan_wi(int NWK) { return NWK > 4 ? 2 : 4; }

template <int NWK, int WI, int NC>
static size_t fast_lds_bytes()
{
    return (size_t)NC * (NWK * 16 + FAST_ROWS_SLACK) * WAVE * sizeof(int32_t) * (WI > 1 ? 2 : 1);
}

template <int NWK, int WI, int NC, bool DUMP, bool COUNT, bool WIDE = false, bool GROUPED = false>
static hipError_t launch_one(hipStream_t st, const FastArgs &a, int grid)
{
    const size_t lds = fast_lds_bytes<NWK, WI, NC>();
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(
            (const void *)recurrence_fast_kernel<NWK, WI, NC, DUMP, COUNT, WIDE, GROUPED>,
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((recurrence_fast_kernel<NWK, WI, NC, DUMP, COUNT, WIDE, GROUPED>), dim3(grid),
                       dim3(WAVE * NWK * WI), lds, st, a.p, a.recs,
                       a.sizes, a.cand, a.n_cand_p, a.ticket, a.wave_relax, a.chunk_min, a.prune,
                       a.descending, a.Fmin, a.Sbest, a.dummy_idx, a.F_all, a.s_top_p, a.group_min,
                       a.grouped);
    return hipGetLastError();
}

template <int NWK>
static hipError_t launch_nwk(hipStream_t st, const FastArgs &a, int mode, int nc, int grid)
{
    switch (mode) {
    case FAST_MODE_PLAN: return launch_one<NWK, plan_wi(NWK), 1, true, false>(st, a, grid);
    case FAST_MODE_COUNT:
        if (a.p.D > WAVE) return launch_one<NWK, 1, 2, false, true, true>(st, a, grid);
        if (a.grouped) return launch_one<NWK, 1, 1, false, true, false, true>(st, a, grid);
        return nc == 2 ? launch_one<NWK, 1, 2, false, true>(st, a, grid)
                       : launch_one<NWK, 1, 1, false, true>(st, a, grid);
    default:
        if (a.p.D > WAVE) return launch_one<NWK, 1, 2, false, false, true>(st, a, grid);
        if (a.grouped) return launch_one<NWK, 1, 1, false, false, false, true>(st, a, grid);
        return nc == 2 ? launch_one<NWK, 1, 2, false, false>(st, a, grid)
                       : launch_one<NWK, 1, 1, false, false>(st, a, grid);
    }
}

template <int NWK, int NC>
static int blocks_per_cu()
{
    int nb = 0;
    const size_t lds = fast_lds_bytes<NWK, 1, NC>();
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)recurrence_fast_kernel<NWK, 1, NC, false, false>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
        &nb, recurrence_fast_kernel<NWK, 1, NC, false, false>, WAVE * NWK, lds);
    return e == hipSuccess ? nb : 0;
}

}  // namespace alpa
