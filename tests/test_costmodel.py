"""ds_cost_table_build against the oracle (host code: bit-exact), and the planner on profiled-style tables."""
import numpy as np
import pytest

from oracle import costmodel as ocm
from oracle import plan as oplan
from paper_2311_10418_amd import binding as ds

INF = 1 << 50


def _rand_grid(rng, nb, nl, holes=0):
    b = np.cumsum(rng.integers(1, 4, nb)).astype(np.int32)
    l = np.cumsum(rng.integers(1, 40, nl)).astype(np.int32)
    t = rng.uniform(0.0, 5000.0, size=(nb, nl))
    for _ in range(holes):
        t[rng.integers(nb), rng.integers(nl)] = np.nan
    return b, l, t


@pytest.mark.parametrize("seed", range(6))
def test_table_is_bit_exact_against_the_oracle(seed):
    rng = np.random.default_rng(seed)
    nb, nl = int(rng.integers(1, 6)), int(rng.integers(1, 7))
    b, l, t = _rand_grid(rng, nb, nl, holes=seed % 3)
    tb, tl = int(b[-1]) + 2, int(l[-1]) + 3                    # a margin beyond the grid
    scale = [1.0, 1000.0, 0.37, 1e6][seed % 4]
    got = ds.ds_cost_table_build(b, l, t, tb, tl, scale=scale, inf_cost=INF)
    ref = ocm.build_table(b, l, t, tb, tl, scale, INF).reshape(tb, tl)
    assert np.array_equal(got, ref)


def test_power_of_two_grid_of_a_launch_bound_machine():
    # t = fixed launch cost + work term: what a profile of small micro-batches looks like
    b = [1, 2, 4, 8, 16, 32]
    l = [16, 32, 64, 128, 256, 512]
    t = np.array([[1500.0 + 0.02 * bb * ll * (1 + ll / 2048.0) for ll in l] for bb in b])
    for bi, bb in enumerate(b):
        for li, ll in enumerate(l):
            if bb * ll > 4096:
                t[bi, li] = np.nan
    got = ds.ds_cost_table_build(b, l, t, 32, 512, scale=1000.0, inf_cost=INF)
    ref = ocm.build_table(b, l, t, 32, 512, 1000.0, INF).reshape(32, 512)
    assert np.array_equal(got, ref)
    # and the planner, fed that table, reproduces the oracle's partition on a seeded batch
    rng = np.random.default_rng(11)
    lens = np.clip(np.rint(rng.lognormal(4.0, 0.8, 48)), 8, 512).astype(np.int32)
    cm = ds.make_cost_model(kind=ds.DS_COST_TABLE, table=got)
    lay = ds.dp_plan(lens, cm, 1024, 4)
    o = oplan.plan(lens, 1024, 4, kind=oplan.COST_TABLE, table=got)
    assert np.array_equal(lay.perm, o["perm"]) and np.array_equal(lay.cuts, o["cuts"])
    assert lay.objective == o["objective"] and lay.t_max == o["t_max"]
    assert lay.n_mb < len(lens)                                # the fixed cost makes merging pay


@pytest.mark.parametrize("bad", ["unsorted", "neg_time", "scale", "overflow", "empty"])
def test_errors(bad):
    b, l = [1, 2, 4], [16, 32]
    t = np.ones((3, 2))
    kw = dict(scale=1.0, inf_cost=INF)
    if bad == "unsorted":
        b = [1, 4, 2]
    elif bad == "neg_time":
        t[1, 1] = -1.0
    elif bad == "scale":
        kw["scale"] = 0.0
    elif bad == "overflow":
        kw["inf_cost"] = 1
    elif bad == "empty":
        b, t = [], np.ones((0, 2))
    with pytest.raises(ds.DsError) as e:
        ds.ds_cost_table_build(b, l, t, 4, 32, **kw)
    assert e.value.code == (ds.DS_EOVERFLOW if bad == "overflow" else ds.DS_EINVAL)
