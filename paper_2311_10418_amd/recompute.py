"""Dynamic recomputation on this build's own stage (GPU report).

The paper (section "Implementation", paragraph "Dynamic recomputation") picks, for every iteration, the
recomputation scheme with the least overhead that stays inside the memory limit, by repeating micro-batch
construction and scheduling under each scheme's cost model.  This module measures the two schemes the HIP
stage offers on a seeded batch (time of one forward + backward over the whole batch and device workspace,
keeping every activation against full recomputation), turns the measurements into two cost models
(the polynomial t(b, L) scaled to each scheme's measured time, in nanoseconds) and activation sizes (bytes
of workspace per padded row), and lets ds_plan_recompute choose under a range of memory limits.

    python -m paper_2311_10418_amd.recompute --config gpt_2048_bf16        # one JSON report on stdout

All arithmetic of the method runs in the library; this file generates inputs, calls it and reads the clock.
"""
import argparse
import json
import sys

import numpy as np

from . import binding as ds
from . import workload as wl
from .costmodel import StageRunner

MODES = (("none", ds.DS_RECOMPUTE_NONE), ("full", ds.DS_RECOMPUTE_FULL))


def poly_table(scale, tb, tl, lin=2048):
    """int64 [tb, tl]: round(scale * b * L * (lin + L)) for b = 1..tb, L = 1..tl."""
    b = np.arange(1, tb + 1, dtype=np.float64)[:, None]
    L = np.arange(1, tl + 1, dtype=np.float64)[None, :]
    return np.rint(scale * b * L * (lin + L)).astype(np.int64)


def report(config="gpt_2048_bf16", seed=0, reps=5, log=None):
    cfg = wl.CONFIGS[config]
    if cfg["kind"] != "gpt":
        raise SystemExit("the report covers decoder-only stages")
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=seed)
    c, cap = cfg["num_stages"], cfg["cap"]
    layout = ds.dp_plan(lens, ds.make_cost_model(), cap, c)
    R = int(layout.total_rows)
    units = float(sum(int(x) for x in layout.mb_cost))          # sum of b * L * (2048 + L) over the plan's micro-batches
    d, F, Ln, H = cfg["d_model"], cfg["d_ff"], cfg["n_layers"], cfg["n_heads"]
    code = ds.DS_DTYPE_BF16 if cfg["dtype"] == "bf16" else ds.DS_DTYPE_F32
    measured = {}
    for name, mode in MODES:
        runner = StageRunner(cfg, max_rows=R, max_seqs=len(lens), seed=seed, recompute=mode)
        ms = runner.time_ms(lambda: runner.run(layout), reps=reps, warmup=2)
        need = [ds.ds_stage_workspace_need(ds.DS_MODEL_GPT, code, Ln, d, H, F, max_rows=r, max_seqs=len(lens), recompute=mode)
                for r in (R // 2, R)]
        measured[name] = {"ms_per_step": ms, "workspace_bytes": int(runner.stage.workspace_bytes()),
                          "workspace_bytes_per_row": (need[1] - need[0]) / float(R - R // 2)}
        assert measured[name]["workspace_bytes"] == need[1]
        if log:
            log("%s: %.2f ms, workspace %.2f GB" % (name, ms, need[1] / 2 ** 30))
        runner.close()
    # cost models in nanoseconds: the polynomial's shape, each scheme's measured scale
    tb = int(len(lens))
    tl = int(lens.max())
    schemes, tables = [], []
    for name, _ in MODES:
        scale = measured[name]["ms_per_step"] * 1e6 / units
        tab = poly_table(scale, tb, tl)
        tables.append(tab)
        # forward share: one forward of three equal parts when nothing is recomputed; full recomputation adds
        # (layers - 1) / layers of a forward to the backward
        fwd = (1, 3) if name == "none" else (Ln, 4 * Ln - 1)
        schemes.append((ds.make_cost_model(kind=ds.DS_COST_TABLE, table=tab), int(round(measured[name]["workspace_bytes_per_row"])),
                        fwd[0], fwd[1]))
    a_none, a_full = schemes[0][1], schemes[1][1]
    limits = sorted({a_full * tl + 1, (a_full * tl + a_none * tl) // 2, a_none * tl + 1, a_none * cap // 4, a_none * cap // 2,
                     a_none * cap + 1, 4 * a_none * cap, a_none * R})
    sweep = []
    for lim in limits:
        try:
            chosen, lay, ms, pk = ds.ds_plan_recompute(lens, schemes, int(lim), c)
            sweep.append({"mem_limit_gb": lim / 2 ** 30, "chosen": MODES[chosen][0], "n_micro_batches": int(lay.n_mb),
                          "makespan_ms": [None if v < 0 else round(float(v) / 1e6, 3) for v in ms],
                          "peak_gb": [None if v < 0 else round(float(v) / 2 ** 30, 3) for v in pk]})
        except ds.DsError as e:
            sweep.append({"mem_limit_gb": lim / 2 ** 30, "chosen": None, "error": str(e)})
    return {"config": config, "n_seq": int(len(lens)), "rows": R, "num_stages": c, "measured": measured,
            "overhead_of_full_recomputation": measured["full"]["ms_per_step"] / measured["none"]["ms_per_step"],
            "workspace_ratio_full_over_none": measured["full"]["workspace_bytes"] / measured["none"]["workspace_bytes"],
            "activation_bytes_per_row": {"none": a_none, "full": a_full}, "limit_sweep": sweep}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gpt_2048_bf16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    rep = report(args.config, args.seed, args.reps, log=lambda *a: print(*a, file=sys.stderr, flush=True))
    print(json.dumps(rep), flush=True)


if __name__ == "__main__":
    main()
