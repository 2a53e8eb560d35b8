"""CPU oracle for the physical placement of a plan's submeshes.

TEST INFRASTRUCTURE ONLY (tests, the smoke check and the benchmark's cpu-baseline leg); shares
nothing with the HIP library.

What is followed (Sec. 5.2, the sentences after the submesh-shape reduction, and the proof in
Appendix A): devices are given to larger submeshes first and then to smaller ones; stages of one
shape that are neighbours in the pipeline are put next to each other.  Appendix A's argument is
used constructively: whole-row submeshes (n, M) are stacked first, then the one-row submeshes
(1, 2^p), which tile the remaining rows because their sizes are powers of two dividing M.

Readings taken where the paper is silent:
  - "larger first" is by device count, descending; equal counts keep pipeline order (this is
    what puts neighbouring stages of one shape side by side);
  - positions are handed out in row-major order from row 0, column 0;
  - (1, M) counts as a one-row submesh; it is smaller than every (n, M) with n >= 2.
The mesh is an N x M grid of cells; a stage's submesh is the rectangle
rows [row, row + n) x columns [col, col + m).

Pins (tests marked "not gpu"): the result is a partition of the grid into rectangles of the
requested shapes with one-row submeshes aligned to their size (Appendix A), whole-row
submeshes occupy the top rows, equal shapes appear in pipeline order along the row-major scan,
and an exhaustive check over every shape multiset of small meshes.
"""


def place(N, M, stage_shapes):
    """stage_shapes: list of (n, m) in pipeline order.  Returns a list of (row, col)."""
    grid = [[None] * M for _ in range(N)]
    by_size = sorted(range(len(stage_shapes)),
                     key=lambda p: (-stage_shapes[p][0] * stage_shapes[p][1], p))
    out = [None] * len(stage_shapes)
    for p in by_size:
        n, m = stage_shapes[p]
        # first free cell in row-major order
        spot = next(((r, c) for r in range(N) for c in range(M) if grid[r][c] is None), None)
        if spot is None:
            raise ValueError("more devices requested than the mesh has")
        r0, c0 = spot
        for r in range(r0, r0 + n):
            for c in range(c0, c0 + m):
                if r >= N or c >= M or grid[r][c] is not None:
                    raise ValueError("submesh does not fit at the scan position")
                grid[r][c] = p
        out[p] = (r0, c0)
    if any(cell is None for row in grid for cell in row):
        raise ValueError("the submeshes do not cover the mesh")
    return out
