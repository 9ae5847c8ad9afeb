"""dp_plan_replicas / ds_assign_replicas against the oracle: host code, bit-exact."""
import numpy as np
import pytest

from oracle import plan as oplan
from oracle import replicas as orep
from paper_2311_10418_amd import binding as ds


@pytest.mark.parametrize("seed", range(25))
def test_assignment_is_bit_exact(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(0, 60))
    k = int(rng.integers(1, 9))
    hi = [4, 50, 10 ** 6, 10 ** 12][seed % 4]                 # small ranges force ties
    t = [int(x) for x in rng.integers(0, hi, n)]
    rep, sums = ds.ds_assign_replicas(t, k)
    orep_of, osums = orep.karmarkar_karp(t, k)
    assert list(rep) == orep_of and list(sums) == osums


@pytest.mark.parametrize("seed", range(12))
def test_plan_with_replicas_is_bit_exact(seed):
    rng = np.random.default_rng(50 + seed)
    n = int(rng.integers(1, 40))
    lens = np.clip(np.rint(rng.lognormal(4.0, 0.9, n)), 4, 512).astype(np.int32)
    c, D = int(rng.integers(1, 6)), int(rng.integers(1, 9))
    cap = int(rng.integers(int(lens.max()), 6 * int(lens.max())))
    fixed = [0, 3000, 100000][seed % 3]
    lay, rep, sums = ds.dp_plan_replicas(lens, ds.make_cost_model(fixed=fixed, lin=256), cap, c, D)
    o = orep.plan_replicas(lens, cap, c, D, fixed=fixed, lin=256)
    assert np.array_equal(lay.perm, o["perm"]) and np.array_equal(lay.cuts, o["cuts"])
    assert lay.objective == o["objective"] and lay.t_max == o["t_max"]
    assert list(lay.mb_cost) == o["mb_cost"]
    assert list(rep) == o["replica_of_mb"] and list(sums) == o["replica_time"]
    # the paper's upper bound of the hybrid iteration time, and its lower bound used in the planner
    upper = (c - 1) * int(lay.t_max) + int(sums.max())
    assert upper * D >= lay.objective
    assert int(sums.sum()) == int(lay.mb_cost.sum())


def test_encoder_decoder_and_table_costs():
    rng = np.random.default_rng(7)
    lens = rng.integers(8, 200, 20).astype(np.int32)
    tgts = rng.integers(1, 60, 20).astype(np.int32)
    lay, rep, sums = ds.dp_plan_replicas(lens, ds.make_cost_model(kind=ds.DS_COST_POLY_T5, fixed=5000), 800, 4, 3, lengths_tgt=tgts)
    o = orep.plan_replicas(lens, 800, 4, 3, lengths_tgt=tgts, kind=oplan.COST_POLY_T5, fixed=5000)
    assert np.array_equal(lay.cuts, o["cuts"]) and list(rep) == o["replica_of_mb"] and list(sums) == o["replica_time"]
    table = (1000 + np.arange(1, 21)[:, None] * np.arange(1, 201)[None, :] * 3).astype(np.int64)
    lay, rep, sums = ds.dp_plan_replicas(lens, ds.make_cost_model(kind=ds.DS_COST_TABLE, table=table), 800, 2, 4)
    o = orep.plan_replicas(lens, 800, 2, 4, kind=oplan.COST_TABLE, table=table)
    assert np.array_equal(lay.cuts, o["cuts"]) and list(rep) == o["replica_of_mb"] and list(sums) == o["replica_time"]


def test_one_replica_is_the_plain_plan():
    rng = np.random.default_rng(9)
    lens = rng.integers(8, 300, 30).astype(np.int32)
    cm = ds.make_cost_model(fixed=20000)
    a = ds.dp_plan(lens, cm, 1024, 4)
    b, rep, sums = ds.dp_plan_replicas(lens, cm, 1024, 4, 1)
    assert np.array_equal(a.cuts, b.cuts) and a.objective == b.objective
    assert np.all(rep == 0) and sums[0] == int(a.mb_cost.sum())


def test_errors():
    cm = ds.make_cost_model()
    with pytest.raises(ds.DsError) as e:
        ds.dp_plan_replicas([10, 20], cm, 100, 4, 0)
    assert e.value.code == ds.DS_EINVAL
    with pytest.raises(ds.DsError) as e:
        ds.ds_assign_replicas([5, -1], 2)
    assert e.value.code == ds.DS_EINVAL
    with pytest.raises(ds.DsError) as e:
        ds.ds_assign_replicas([2 ** 62, 2 ** 62], 2)
    assert e.value.code == ds.DS_EOVERFLOW
    with pytest.raises(ds.DsError) as e:
        ds.dp_plan_replicas([10, 200], cm, 100, 4, 2)           # a sequence alone exceeds the cap
    assert e.value.code == ds.DS_EINFEASIBLE
