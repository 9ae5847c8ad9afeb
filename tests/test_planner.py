"""Host planner (dp_plan in libdynastage.so) against the partition oracle: identical order,
identical cuts, identical objective and t_max, identical error class.  CPU only."""
import numpy as np
import pytest

from oracle import plan as oplan
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl


def _same(lens, cap, c, tgts=None, kind=0, fixed=0, lin=2048, table=None):
    cm = ds.make_cost_model(kind=kind, fixed=fixed, lin=lin, table=table)
    try:
        ref = oplan.plan(lens, cap, c, lengths_tgt=tgts, kind=kind, fixed=fixed, lin=lin, table=table)
    except oplan.OraclePlanError as e:
        with pytest.raises(ds.DsError) as g:
            ds.dp_plan(lens, cm, cap, c, lengths_tgt=tgts)
        assert g.value.code == e.code
        return None
    lo = ds.dp_plan(lens, cm, cap, c, lengths_tgt=tgts)
    assert list(lo.perm) == list(ref["perm"])
    assert list(lo.cuts) == list(ref["cuts"])
    assert lo.objective == ref["objective"]
    assert lo.t_max == ref["t_max"]
    return lo


def test_random_small_cases_table_costs():
    rng = np.random.default_rng(21)
    for _ in range(3000):
        n = int(rng.integers(1, 13))
        lmax = int(rng.integers(1, 10))
        lens = rng.integers(1, lmax + 1, size=n).astype(np.int32)
        table = rng.integers(1, 50, size=(n, lmax)).astype(np.int64)
        cap = int(rng.integers(1, 5 * lmax + 1))
        c = int(rng.choice([1, 2, 4, 8]))
        _same(lens, cap, c, kind=ds.DS_COST_TABLE, table=table)


def test_random_poly_costs_with_fixed_term():
    rng = np.random.default_rng(22)
    for _ in range(300):
        n = int(rng.integers(1, 70))
        lens = np.clip(np.rint(rng.lognormal(4.0, 1.0, size=n)), 1, 600).astype(np.int32)
        fixed = int(rng.choice([0, 1000, 50000, 10 ** 6]))
        cap = int(rng.choice([600, 2048, 4096]))
        c = int(rng.choice([1, 2, 4, 8]))
        _same(lens, cap, c, fixed=fixed, lin=int(rng.choice([1, 64, 2048])))


def test_random_encoder_decoder_costs():
    rng = np.random.default_rng(23)
    for _ in range(200):
        n = int(rng.integers(1, 50))
        lens = np.clip(np.rint(rng.lognormal(4.0, 1.0, size=n)), 1, 400).astype(np.int32)
        tgts = np.clip(np.rint(rng.lognormal(2.5, 1.0, size=n)), 1, 100).astype(np.int32)
        fixed = int(rng.choice([0, 2000, 10 ** 5]))
        _same(lens, int(rng.choice([400, 2048])), int(rng.choice([1, 4])), tgts=tgts, kind=ds.DS_COST_POLY_T5, fixed=fixed)


@pytest.mark.parametrize("name", ["gpt_small_fp32", "gpt_2048_bf16", "t5_1024_bf16", "gpt_4096_longtail_bf16"])
def test_named_configurations(name):
    cfg = wl.CONFIGS[name]
    lens, tgts = wl.draw_lengths(cfg["lengths"], seed=0)
    kind = ds.DS_COST_POLY_T5 if cfg["kind"] == "t5" else ds.DS_COST_POLY_GPT
    lo = _same(lens, cfg["cap"], cfg["num_stages"], tgts=tgts, kind=kind)
    # closed form for a cost without a fixed term: zero padding, J = (c-1) g(max) + sum g
    assert lo.total_rows == lo.total_tokens == int(lens.sum())
    if cfg["kind"] == "gpt":
        g = lambda l: int(l) * (2048 + int(l))
        assert lo.objective == (cfg["num_stages"] - 1) * g(lens.max()) + sum(g(l) for l in lens)
    # and with a per-micro-batch overhead, where merging pays off and the cap binds
    _same(lens, cfg["cap"], cfg["num_stages"], tgts=tgts, kind=kind, fixed=2_000_000)


def test_error_codes():
    cm = ds.make_cost_model()
    for lens, cap, c, code in (([0, 4], 10, 4, ds.DS_EINVAL), ([4, 50], 49, 4, ds.DS_EINFEASIBLE),
                               ([3], 10, 0, ds.DS_EINVAL), ([3], 0, 2, ds.DS_EINVAL)):
        with pytest.raises(ds.DsError) as e:
            ds.dp_plan(lens, cm, cap, c)
        assert e.value.code == code
    with pytest.raises(ds.DsError) as e:
        ds.dp_plan([2 ** 30, 2 ** 30], ds.make_cost_model(lin=2 ** 62), 2 ** 40, 4)
    assert e.value.code == ds.DS_EOVERFLOW
    with pytest.raises(ds.DsError) as e:
        ds.dp_plan([3, 4], None, 10, 2)
    assert e.value.code == ds.DS_EINVAL
    with pytest.raises(ds.DsError) as e:          # encoder-decoder cost without target lengths
        ds.dp_plan([3, 4], ds.make_cost_model(kind=ds.DS_COST_POLY_T5), 10, 2)
    assert e.value.code == ds.DS_EINVAL


def test_layout_tables():
    lens = np.array([5, 3, 9, 3, 7], dtype=np.int32)
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=10 ** 6, lin=1), 18, 2)
    # rows: every sequence inside its micro-batch block, blocks back to back, padded to the longest
    srt = lens[lo.perm]
    row = 0
    for m in range(lo.n_mb):
        a, b = lo.mb_start[m], lo.mb_start[m] + lo.mb_count[m]
        assert lo.mb_lpad[m] == srt[a:b].max()
        assert lo.mb_row[m] == row and lo.mb_nrows[m] == lo.mb_count[m] * lo.mb_lpad[m]
        for j, s in enumerate(range(a, b)):
            assert lo.seq_row[s] == row + j * lo.mb_lpad[m] and lo.seq_len[s] == srt[s]
        row += lo.mb_nrows[m]
        assert lo.mb_count[m] * lo.mb_lpad[m] <= 18
    assert lo.total_rows == row and lo.total_tokens == lens.sum()
    # padding efficiency = non-pad tokens / processed tokens (section "Background")
    assert 0 < lo.total_tokens / lo.total_rows <= 1


def test_baseline_layouts():
    lens = np.array([5, 3, 9, 3, 7, 2], dtype=np.int32)
    fixed = ds.ds_layout_from_cuts(lens, [0, 2, 4, 6], pad_to=9)
    assert fixed.total_rows == 6 * 9 and list(fixed.mb_lpad) == [9, 9, 9]
    assert list(fixed.seq_row) == [0, 9, 18, 27, 36, 45]
    packed = ds.ds_layout_packed(lens, 10, 2)
    # first fit into rows of 10: row0 = [5,3,2], row1 = [9], row2 = [3,7]
    by_orig = {int(packed.perm[s]): (int(packed.seq_row[s]), int(packed.seq_len[s])) for s in range(6)}
    assert by_orig == {0: (0, 5), 1: (5, 3), 5: (8, 2), 2: (10, 9), 3: (20, 3), 4: (23, 7)}
    assert packed.n_mb == 2 and packed.total_rows == 40 and list(packed.mb_count) == [4, 2]
    single = ds.ds_layout_from_cuts(lens, list(range(7)))
    assert single.total_rows == lens.sum() and single.n_mb == 6
    with pytest.raises(ds.DsError):
        ds.ds_layout_from_cuts(lens, [0, 3, 3, 6])
    with pytest.raises(ds.DsError):
        ds.ds_layout_packed(lens, 8, 2)


def test_planner_is_reentrant():
    import concurrent.futures
    lens, _ = wl.draw_lengths(wl.CONFIGS["gpt_2048_bf16"]["lengths"], seed=3)
    cm = ds.make_cost_model(fixed=500000)

    def run(_):
        lo = ds.dp_plan(lens, cm, 16384, 4)
        return lo.objective, tuple(lo.cuts)

    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        res = list(ex.map(run, range(8)))
    assert len(set(res)) == 1
