"""Full recomputation on the GPU: the stage with DS_RECOMPUTE_FULL gives bit-identical results to the stage that keeps
every activation (same kernels on the same inputs, run again), matches the oracle to the same bar, and holds one
layer's activations instead of all layers'.  Paper: section "Implementation", paragraph "Dynamic recomputation"."""
import numpy as np
import pytest
import torch

from oracle import stage as ost
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl
from helpers import check, check_seqs, run_gpt_stage, run_t5_stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype_code", [ds.DS_DTYPE_F32, ds.DS_DTYPE_BF16])
def test_gpt_recompute_is_bit_identical_and_matches_oracle(dtype_code):
    bf16 = dtype_code == ds.DS_DTYPE_BF16
    cfg = dict(wl.CONFIGS["gpt_small_fp32"])
    cfg["n_layers"] = 3                                     # a first, a middle and a last layer
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=4)
    lens = lens[:40]
    params = wl.draw_params(wl.GPT_KEYS, 3, cfg["d_model"], cfg["d_ff"], seed=4, bf16=bf16)
    xs = wl.draw_embedded_tokens(lens, cfg["d_model"], seed=4, bf16=bf16)
    dys = wl.draw_rows(lens, cfg["d_model"], seed=4, tag=5, bf16=bf16)
    ref = ost.gpt_stage_fwd_bwd(xs, dys, params, cfg["n_heads"])
    tol = 2e-2 if bf16 else 1e-4
    for name, lo in (("dp_overhead", ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cfg["cap"], 4)),
                     ("singletons", ds.ds_layout_from_cuts(lens, list(range(len(lens) + 1))))):
        keep = run_gpt_stage(lo, cfg, params, xs, dys, dtype_code)
        redo = run_gpt_stage(lo, cfg, params, xs, dys, dtype_code, recompute=ds.DS_RECOMPUTE_FULL)
        for a, b in zip(keep[0] + keep[1], redo[0] + redo[1]):
            assert np.array_equal(a, b), name
        for ga, gb in zip(keep[2], redo[2]):
            for k in ga:
                assert np.array_equal(ga[k], gb[k]), (name, k)
        check_seqs(redo[0], ref[0], tol, name + " act_out")
        check_seqs(redo[1], ref[1], tol, name + " grad_in")
        for li, layer in enumerate(ref[2]):
            for k, v in layer.items():
                check(redo[2][li][k], v, tol, "%s L%d.%s" % (name, li, k))
        assert redo[3].size == 0 or np.all(redo[3] == 0)


def test_t5_recompute_is_bit_identical():
    import test_gpu_stage_t5 as t5
    lens, tgts, ep, dp, ex, dx, ddy = t5._case(True)
    cfg = dict(t5.CFG)
    cm = ds.make_cost_model(kind=ds.DS_COST_POLY_T5, fixed=1_500_000)
    lo = ds.dp_plan(lens, cm, 2048, 4, lengths_tgt=tgts)
    keep = run_t5_stage(lo, cfg, ep, dp, ex, dx, ddy, ds.DS_DTYPE_BF16)
    redo = run_t5_stage(lo, cfg, ep, dp, ex, dx, ddy, ds.DS_DTYPE_BF16, recompute=ds.DS_RECOMPUTE_FULL)
    for key in ("outs", "d_enc", "d_dec"):
        for a, b in zip(keep[key], redo[key]):
            assert np.array_equal(a, b), key
    for key in ("eg", "dg"):
        for ga, gb in zip(keep[key], redo[key]):
            for k in ga:
                assert np.array_equal(ga[k], gb[k]), (key, k)
    r_outs = ost.t5_stage_fwd_bwd(ex, dx, ddy, ep, dp, cfg["n_heads"])[0]
    check_seqs(redo["outs"], r_outs, 2e-2, "dec_out")


def test_workspace_matches_the_host_estimate_and_shrinks():
    args = dict(model=ds.DS_MODEL_GPT, dtype=ds.DS_DTYPE_BF16, n_layers=4, d_model=256, n_heads=2, d_ff=1024, max_rows=3000, max_seqs=20)
    sizes = {}
    for mode in (ds.DS_RECOMPUTE_NONE, ds.DS_RECOMPUTE_FULL):
        st = ds.Stage(recompute=mode, **args)
        sizes[mode] = st.workspace_bytes()
        assert sizes[mode] == ds.ds_stage_workspace_need(recompute=mode, **args)
        st.close()
    assert sizes[ds.DS_RECOMPUTE_FULL] < sizes[ds.DS_RECOMPUTE_NONE]
    torch.cuda.synchronize()
