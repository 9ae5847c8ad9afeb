"""TEST INFRASTRUCTURE: the profiled cost model's time table, written out from its definition.

The paper (section "Overview", paragraph "Cost models") profiles the execution time of a
micro-batch at power-of-two micro-batch sizes and sequence lengths and bridges the gaps by linear
interpolation.  Reading taken here (the paper does not say more):

* interpolation is linear along each axis on the raw (b, L) coordinates, i.e. bilinear inside a
  grid cell: first along b at the two bracketing lengths, then along L between those two values;
* a length below the smallest profiled one costs what the smallest profiled one costs;
* a micro-batch size or length beyond the largest profiled one, and any point whose bracketing
  grid points (those with non-zero weight) include an unprofiled one (NaN), gets `inf_cost`, a
  cost no plan can afford;
* times are turned into integers as floor(t * scale + 0.5), at least 1.

table[(b-1)*tl + (L-1)] for b = 1..tb, L = 1..tl, the layout the planner's table cost model reads.
Plain Python loops over float64 scalars; no blocking, no vectorisation.
"""
import math

import numpy as np


def _bracket(grid, x):
    """Index i with grid[i] <= x <= grid[i+1] and the weight of grid[i+1]; (i, 0.0) when x == grid[i]."""
    n = len(grid)
    for i in range(n):
        if x == grid[i]:
            return i, 0.0
    for i in range(n - 1):
        if grid[i] < x < grid[i + 1]:
            return i, (float(x) - float(grid[i])) / (float(grid[i + 1]) - float(grid[i]))
    raise ValueError("outside the grid")


def interpolate_time(b_grid, l_grid, t, b, L):
    """Interpolated time at (b, L), or None where the definition above gives no value."""
    if b < b_grid[0] or b > b_grid[-1] or L > l_grid[-1]:
        return None
    Lc = max(L, l_grid[0])
    i, u = _bracket(b_grid, b)
    j, v = _bracket(l_grid, Lc)

    def along_b(jj):
        lo = float(t[i][jj])
        if u == 0.0:
            return lo
        hi = float(t[i + 1][jj])
        return lo + u * (hi - lo)

    near = along_b(j)
    if v == 0.0:
        val = near
    else:
        far = along_b(j + 1)
        val = near + v * (far - near)
    return None if math.isnan(val) else val


def build_table(b_grid, l_grid, t, tb, tl, scale, inf_cost):
    b_grid = [int(x) for x in b_grid]
    l_grid = [int(x) for x in l_grid]
    out = np.empty(tb * tl, dtype=np.int64)
    for b in range(1, tb + 1):
        for L in range(1, tl + 1):
            val = interpolate_time(b_grid, l_grid, t, b, L)
            if val is None:
                out[(b - 1) * tl + (L - 1)] = inf_cost
            else:
                out[(b - 1) * tl + (L - 1)] = max(1, int(math.floor(val * float(scale) + 0.5)))
    return out
