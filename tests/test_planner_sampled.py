"""dp_plan_sampled against its oracle (host code, exact) and against dp_plan."""
import time

import numpy as np
import pytest

from oracle import quantized as oq
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl


@pytest.mark.parametrize("seed", range(20))
def test_bit_exact_against_the_oracle(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 30))
    lens = np.clip(np.rint(rng.lognormal(4.0, 0.9, n)), 4, 400).astype(np.int32)
    cap = int(rng.integers(int(lens.max()), 6 * int(lens.max())))
    c, fixed = int(rng.integers(1, 7)), int(rng.integers(0, 60000))
    q = [1, 13, 5000, 250000][seed % 4]
    lay = ds.dp_plan_sampled(lens, ds.make_cost_model(fixed=fixed, lin=128), cap, c, q)
    o = oq.plan(lens, cap, c, q, fixed=fixed, lin=128)
    assert np.array_equal(lay.perm, o["perm"]) and np.array_equal(lay.cuts, o["cuts"])
    assert lay.objective == o["objective"] and lay.t_max == o["t_max"]


def test_table_cost_and_interval_one():
    rng = np.random.default_rng(5)
    lens = rng.integers(8, 150, 25).astype(np.int32)
    table = (3000 + np.arange(1, 26)[:, None] * np.arange(1, 151)[None, :] * 7).astype(np.int64)
    cm = ds.make_cost_model(kind=ds.DS_COST_TABLE, table=table)
    a = ds.dp_plan(lens, cm, 600, 4)
    b = ds.dp_plan_sampled(lens, cm, 600, 4, 1)
    assert np.array_equal(a.cuts, b.cuts) and a.objective == b.objective
    o = oq.plan(lens, 600, 4, 900, table=table)
    s = ds.dp_plan_sampled(lens, cm, 600, 4, 900)
    assert np.array_equal(s.cuts, o["cuts"]) and s.objective == o["objective"]


def test_loss_bound_and_errors_at_the_bench_batch():
    cfg = wl.CONFIGS["gpt_2048_bf16"]
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=0)
    cm = ds.make_cost_model(fixed=3 * 10 ** 6)                    # a per-micro-batch overhead, so that merging pays
    exact = ds.dp_plan(lens, cm, cfg["cap"], cfg["num_stages"])
    for q in (10 ** 4, 10 ** 6, 10 ** 8):
        s = ds.dp_plan_sampled(lens, cm, cfg["cap"], cfg["num_stages"], q)
        assert exact.objective <= s.objective < exact.objective + (cfg["num_stages"] - 1) * q + 1
    with pytest.raises(ds.DsError) as e:
        ds.dp_plan_sampled(lens, cm, cfg["cap"], cfg["num_stages"], 0)
    assert e.value.code == ds.DS_EINVAL
