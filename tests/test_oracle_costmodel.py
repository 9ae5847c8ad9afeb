"""Pins of the cost-table oracle against things it does not compute itself."""
import numpy as np
from scipy.interpolate import RegularGridInterpolator

from oracle import costmodel as ocm

B = [1, 2, 4, 8, 16]
LG = [16, 32, 64, 128, 256]
INF = 1 << 50


def _grid(fn):
    return np.array([[fn(b, l) for l in LG] for b in B], dtype=np.float64)


def test_grid_points_are_reproduced():
    rng = np.random.default_rng(0)
    t = rng.uniform(10, 1000, size=(len(B), len(LG)))
    tab = ocm.build_table(B, LG, t, 16, 256, 1000.0, INF).reshape(16, 256)
    for i, b in enumerate(B):
        for j, l in enumerate(LG):
            assert tab[b - 1, l - 1] == int(np.floor(t[i, j] * 1000.0 + 0.5))


def test_bilinear_function_is_exact():
    # an interpolant that is linear along each axis reproduces a + p*b + q*L + r*b*L; asymmetric
    # coefficients, so swapped axes or a transposed grid cannot pass
    f = lambda b, l: 7 + 3 * b + 11 * l + 5 * b * l
    tab = ocm.build_table(B, LG, _grid(f), 16, 256, 1.0, INF).reshape(16, 256)
    for b in range(1, 17):
        for l in range(16, 257, 7):
            assert tab[b - 1, l - 1] == f(b, l), (b, l)


def test_matches_library_linear_interpolation():
    rng = np.random.default_rng(1)
    t = np.cumsum(np.cumsum(rng.uniform(1, 50, size=(len(B), len(LG))), axis=0), axis=1)
    ref = RegularGridInterpolator((np.array(B, float), np.array(LG, float)), t, method="linear")
    tab = ocm.build_table(B, LG, t, 16, 256, 1.0e3, INF).reshape(16, 256)
    for b in range(1, 17):
        for l in range(16, 257, 5):
            assert abs(tab[b - 1, l - 1] - ref([[b, l]])[0] * 1e3) <= 0.5 + 1e-6


def test_midpoints_are_averages_and_short_lengths_are_flat():
    rng = np.random.default_rng(2)
    t = rng.uniform(10, 1000, size=(len(B), len(LG)))
    tab = ocm.build_table(B, LG, t, 16, 256, 1.0e6, INF).reshape(16, 256)
    assert abs(tab[3 - 1, 64 - 1] - 0.5e6 * (t[1, 2] + t[2, 2])) <= 1          # b = 3 between 2 and 4
    assert abs(tab[4 - 1, 96 - 1] - 0.5e6 * (t[2, 2] + t[2, 3])) <= 1          # L = 96 between 64 and 128
    assert np.all(tab[:, :16] == tab[:, 15:16])                                 # L < 16 costs what L = 16 costs


def test_monotone_grid_gives_monotone_table():
    t = _grid(lambda b, l: 100 + b * l * (1 + l / 64.0))
    tab = ocm.build_table(B, LG, t, 16, 256, 10.0, INF).reshape(16, 256)
    assert np.all(np.diff(tab, axis=0) >= 0) and np.all(np.diff(tab, axis=1) >= 0)


def test_unprofiled_points_and_outside_of_grid():
    t = _grid(lambda b, l: 1.0 + b * l)
    t[4, 4] = np.nan                                        # (16, 256) was not profiled
    tab = ocm.build_table(B, LG, t, 20, 300, 1.0, INF).reshape(20, 300)
    assert tab[16 - 1, 256 - 1] == INF
    assert tab[12 - 1, 200 - 1] == INF                      # inside the cell that touches it
    assert tab[16 - 1, 128 - 1] == 1 + 16 * 128             # on the grid line next to it: not touched
    assert tab[8 - 1, 256 - 1] == 1 + 8 * 256
    assert tab[12 - 1, 128 - 1] == 1 + 12 * 128
    assert np.all(tab[16:, :] == INF) and np.all(tab[:, 256:] == INF)          # beyond the grid
    assert tab.min() >= 1
