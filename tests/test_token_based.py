"""ds_layout_token_based (the paper's TB baseline) against its oracle: order and cuts bit-exact, layout
bookkeeping consistent, error classes."""
import numpy as np
import pytest

from oracle import token_based as otb
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl


def _compare(lens, budget, tgts=None):
    ref = otb.plan(lens, budget, lengths_tgt=tgts)
    if ref is None:
        with pytest.raises(ds.DsError) as e:
            ds.ds_layout_token_based(lens, budget, lengths_tgt=tgts)
        assert e.value.code == ds.DS_EINFEASIBLE
        return None
    lo = ds.ds_layout_token_based(lens, budget, lengths_tgt=tgts)
    assert [int(x) for x in lo.perm] == ref["perm"]
    assert list(lo.cuts) == ref["cuts"]
    # padded to the micro-batch's own longest sample; rows = count x padded length, back to back
    ls = [int(lens[i]) for i in ref["perm"]]
    row = 0
    for m, (a, b) in enumerate(zip(ref["cuts"][:-1], ref["cuts"][1:])):
        assert int(lo.mb_lpad[m]) == max(ls[a:b]) and int(lo.mb_row[m]) == row
        row += (b - a) * max(ls[a:b])
        assert (b - a) * max(ls[a:b]) <= budget
    assert lo.total_rows == row and lo.total_tokens == int(np.sum(lens))
    return lo


@pytest.mark.parametrize("seed", range(60))
def test_random_batches_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 200))
    lens = np.clip(np.rint(rng.lognormal(4.0, 1.0, n)), 1, 1024).astype(np.int32)
    tgts = rng.integers(1, 64, n).astype(np.int32) if seed % 3 == 0 else None
    lo_b = int(lens.max()) if seed % 5 else max(1, int(lens.max()) - 1)       # every fifth case may be infeasible
    budget = int(rng.integers(lo_b, 6 * int(lens.max()) + 1))
    _compare(lens, budget, tgts)


@pytest.mark.parametrize("name", ["gpt_small_fp32", "gpt_2048_bf16", "t5_1024_bf16", "gpt_4096_longtail_bf16"])
def test_named_workloads(name):
    cfg = wl.CONFIGS[name]
    lens, tgts = wl.draw_lengths(cfg["lengths"], seed=0)
    for budget in (cfg["cap"] // 4, cfg["cap"] // 2, cfg["cap"]):
        lo = _compare(lens, budget, tgts)
        if lo is not None:
            assert lo.n_mb >= -(-int(lens.sum()) // budget)          # no micro-batch holds more than the budget


def test_objective_is_reported_under_a_cost_model():
    lens = np.array([3, 1, 2, 5, 4, 4], dtype=np.int32)
    lo = ds.ds_layout_token_based(lens, 8, cost_model=ds.make_cost_model(), num_stages=4)
    assert list(lo.cuts) == [0, 2, 4, 5, 6]
    t = [2 * 2 * (2048 + 2), 2 * 4 * (2048 + 4), 1 * 4 * (2048 + 4), 1 * 5 * (2048 + 5)]
    assert lo.t_max == max(t) and lo.objective == 3 * max(t) + sum(t)


def test_argument_errors():
    lens = np.array([3, 1, 2], dtype=np.int32)
    for bad in (0, -5):
        with pytest.raises(ds.DsError) as e:
            ds.ds_layout_token_based(lens, bad)
        assert e.value.code == ds.DS_EINVAL
    with pytest.raises(ds.DsError) as e:
        ds.ds_layout_token_based(np.array([3, 0], dtype=np.int32), 8)
    assert e.value.code == ds.DS_EINVAL
