// Physical device assignment of the submeshes a plan chose (Sec. 5.2, the paragraph after the
// submesh-shape reduction; Appendix A gives the covering argument this construction follows).
// Host code: at most ALPA_DP_MAX_K stages, no device work.
#include "../../include/alpa_dp.h"

#include <algorithm>
#include <numeric>
#include <string>
#include <vector>

extern "C" __attribute__((visibility("hidden"))) int alpa_dp_set_error_(int code, const char *msg);

extern "C" int alpa_place_submeshes(int N, int M, const alpa_shape_t *stage_shapes, int num_stages,
                                    int32_t *out_row, int32_t *out_col)
{
    auto fail = [](int code, const char *msg) { return alpa_dp_set_error_(code, msg); };
    if (!stage_shapes || !out_row || !out_col) return fail(ALPA_DP_EINVAL, "null argument");
    if (N < 1 || M < 1 || (long long)N * M > ALPA_DP_MAX_DEVICES)
        return fail(ALPA_DP_EINVAL, "N x M out of range");
    if ((M & (M - 1)) != 0) return fail(ALPA_DP_EINVAL, "M must be a power of two");
    if (num_stages < 1 || num_stages > ALPA_DP_MAX_K)
        return fail(ALPA_DP_EINVAL, "num_stages out of range");
    long long devices = 0;
    for (int p = 0; p < num_stages; ++p) {
        const int n = stage_shapes[p].n, m = stage_shapes[p].m;
        const bool one_d = n == 1 && m >= 1 && m <= M && (m & (m - 1)) == 0;
        const bool two_d = m == M && n >= 2 && n <= N;
        if (!one_d && !two_d) return fail(ALPA_DP_EINVAL, "shape outside the submesh family");
        devices += (long long)n * m;
    }
    if (devices != (long long)N * M)
        return fail(ALPA_DP_EINVAL, "the submeshes do not add up to N x M devices");
    // larger submeshes first; equal sizes keep their pipeline order, which puts neighbouring
    // stages of one shape next to each other
    std::vector<int> order(num_stages);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        return stage_shapes[a].n * stage_shapes[a].m > stage_shapes[b].n * stage_shapes[b].m;
    });
    // Row-major cursor.  Whole-row submeshes come first (each is larger than any one-row
    // submesh), so they start at column 0; after them the sizes are non-increasing powers of
    // two dividing M, so the cursor's column is always a multiple of the next size and no
    // submesh straddles a row.
    int row = 0, col = 0;
    for (int p : order) {
        const int n = stage_shapes[p].n, m = stage_shapes[p].m;
        if (col % m != 0 || col + m > M || row + n > N)
            return fail(ALPA_DP_EHIP, "internal inconsistency in the placement");
        out_row[p] = row;
        out_col[p] = col;
        col += m;
        if (n > 1) { row += n; col = 0; }
        else if (col == M) { ++row; col = 0; }
    }
    return ALPA_DP_OK;
}
