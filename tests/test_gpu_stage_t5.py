"""GPU parity of the encoder-decoder (T5-style) stage against the per-sequence float64 oracle:
RMSNorm, gated-GELU MLP, bidirectional / causal / cross attention, two token streams, on a DP plan
with a per-micro-batch overhead (padding in both streams, NaN planted in it) and on single-sample
micro-batches.  fp32 runs the generic kernels, bf16 the matrix-core kernels."""
import numpy as np
import pytest

from oracle import stage as ost
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl
from helpers import check, check_seqs, run_t5_stage

pytestmark = pytest.mark.gpu

CFG = dict(d_model=256, n_heads=4, d_ff=512, n_layers=2, n_dec_layers=2)
SPEC = dict(rule="count", count=24, mu=4.2, sigma=0.8, lo=8, hi=300, tgt_mu=3.0, tgt_sigma=0.9, tgt_lo=1, tgt_hi=150)


def _case(bf16):
    lens, tgts = wl.draw_lengths(SPEC, seed=2)
    ep = wl.draw_params(wl.T5_ENC_KEYS, CFG["n_layers"], CFG["d_model"], CFG["d_ff"], seed=2, tag=6, bf16=bf16, std=0.05)
    dp = wl.draw_params(wl.T5_DEC_KEYS, CFG["n_dec_layers"], CFG["d_model"], CFG["d_ff"], seed=2, tag=7, bf16=bf16, std=0.05)
    ex = wl.draw_rows(lens, CFG["d_model"], seed=2, tag=3, bf16=bf16)
    dx = wl.draw_rows(tgts, CFG["d_model"], seed=2, tag=8, bf16=bf16)
    ddy = wl.draw_rows(tgts, CFG["d_model"], seed=2, tag=5, bf16=bf16)
    return lens, tgts, ep, dp, ex, dx, ddy


@pytest.mark.parametrize("dtype_code", [ds.DS_DTYPE_F32, ds.DS_DTYPE_BF16])
def test_t5_stage_matches_oracle(dtype_code):
    bf16 = dtype_code == ds.DS_DTYPE_BF16
    tol = 2e-2 if bf16 else 1e-4
    lens, tgts, ep, dp, ex, dx, ddy = _case(bf16)
    r_outs, r_denc, r_ddec, r_eg, r_dg = ost.t5_stage_fwd_bwd(ex, dx, ddy, ep, dp, CFG["n_heads"])
    cm = ds.make_cost_model(kind=ds.DS_COST_POLY_T5, fixed=1_500_000)
    layouts = [("dp_overhead", ds.dp_plan(lens, cm, 2048, 4, lengths_tgt=tgts)),
               ("singletons", ds.ds_layout_from_cuts(lens, list(range(len(lens) + 1)), lengths_tgt=tgts))]
    assert layouts[0][1].total_rows > layouts[0][1].total_tokens          # the plan really pads
    for name, lo in layouts:
        got = run_t5_stage(lo, CFG, ep, dp, ex, dx, ddy, dtype_code)
        # every sample on its own, every weight-gradient tensor; normwise and elementwise (helpers.check)
        errs = {"dec_out": check_seqs(got["outs"], r_outs, tol, name + " dec_out"),
                "d_enc_in": check_seqs(got["d_enc"], r_denc, tol, name + " d_enc_in"),
                "d_dec_in": check_seqs(got["d_dec"], r_ddec, tol, name + " d_dec_in")}
        for tag, gg, rr in (("enc", got["eg"], r_eg), ("dec", got["dg"], r_dg)):
            for li, layer in enumerate(rr):
                for k, v in layer.items():
                    errs["%s%d.%s" % (tag, li, k)] = check(gg[li][k], v, tol, "%s %s%d.%s" % (name, tag, li, k))
        worst = max(errs, key=errs.get)
        print(name, "worst", worst, "%.3e" % errs[worst])
        for p in got["pads"]:
            assert p.size == 0 or np.all(p == 0), name
