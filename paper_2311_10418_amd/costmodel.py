"""Profiled cost model t(b, L) of this build's own stage, and its check against measurement.

The paper (section "Overview", paragraph "Cost models") profiles the forward+backward time of a
micro-batch at power-of-two micro-batch sizes and sequence lengths on one GPU and bridges the gaps by
linear interpolation; the planner then minimises Eq1 under that model, and section "Accuracy of cost
models" compares predicted with measured iteration times.  This module does the same for the HIP
stage of this package (decoder-only stages):

    profile_grid()    times stage_fwd_bwd on single-micro-batch layouts (b sequences padded to L)
    build_table()     ds_cost_table_build -> the int64 table of a DS_COST_TABLE cost model (nanoseconds)
    report()          plans a seeded batch with the polynomial and with the profiled model, runs every
                      micro-batch of each plan as its own stage call (the way a pipeline stage executes
                      them, one after another) and compares predicted with measured times

    python -m paper_2311_10418_amd.costmodel --config gpt_2048_bf16        # one JSON report on stdout

All arithmetic of the method (interpolation, planning, the stage) runs in the library; this file only
generates inputs, calls it and reads the clock.
"""
import argparse
import json
import sys

import numpy as np

from . import binding as ds
from . import workload as wl

INF_COST = 1 << 50
NS_PER_MS = 1.0e6


def power_of_two_grid(lo, hi):
    """lo, 2*lo, ... up to the first value >= hi."""
    g, v = [], int(lo)
    while True:
        g.append(v)
        if v >= hi:
            return g
        v *= 2


class StageRunner:
    """A GPT stage with seeded random weights and row buffers; runs any layout on a row range."""

    def __init__(self, cfg, max_rows, max_seqs, seed=0, device="cuda:0", recompute=0, same_weights=False):
        import torch
        self.torch = torch
        d, F, L, H = cfg["d_model"], cfg["d_ff"], cfg["n_layers"], cfg["n_heads"]
        bf16 = cfg["dtype"] == "bf16"
        tdt = torch.bfloat16 if bf16 else torch.float32
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        shapes = {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (d, 3 * d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
                  "ln2_g": (d,), "ln2_b": (d,), "w_1": (d, F), "b_1": (F,), "w_2": (F, d), "b_2": (d,)}
        self.weights, self.grads = [], []
        for _ in range(L):
            w, g = {}, {}
            for k in ds.GPT_KEYS:
                v = torch.randn(shapes[k], generator=gen, device=device, dtype=torch.float32) * 0.02
                if k.endswith("_g"):
                    v = v + 1.0
                w[k] = v.to(tdt).contiguous()
                g[k] = torch.zeros(shapes[k], device=device, dtype=torch.float32)
            self.weights.append(w)
            self.grads.append(g)
        self.x = torch.randn((max_rows, d), generator=gen, device=device, dtype=torch.float32).to(tdt)
        self.dy = torch.randn((max_rows, d), generator=gen, device=device, dtype=torch.float32).to(tdt)
        self.out = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16 if bf16 else ds.DS_DTYPE_F32, L, d, H, F,
                              max_rows=max_rows, max_seqs=max_seqs, recompute=recompute)
        if same_weights:
            # every call is a micro-batch of one iteration: the stage keeps its transposed weight copies
            self.stage.weights_unchanged(True)

    def run(self, layout, row0=0, accumulate=False):
        r1 = row0 + layout.total_rows
        if r1 > self.x.shape[0]:
            raise ValueError("layout needs rows up to %d, the runner holds %d" % (r1, self.x.shape[0]))
        ds.stage_fwd_bwd(self.stage, layout, self.weights, self.x[row0:r1], self.dy[row0:r1], self.out[row0:r1],
                         self.dx[row0:r1], self.grads, accumulate=accumulate)

    def time_ms(self, fn, reps=3, warmup=1):
        """Median over `reps` of the time of fn() on the current stream, milliseconds."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    def close(self):
        self.stage.close()


def profile_grid(runner, b_grid, l_grid, max_rows, reps=3, log=None):
    """t[i, j] = milliseconds of one stage call on b_grid[i] sequences of length l_grid[j]; NaN where b*L > max_rows."""
    t = np.full((len(b_grid), len(l_grid)), np.nan)
    for i, b in enumerate(b_grid):
        for j, L in enumerate(l_grid):
            if b * L > max_rows:
                continue
            lay = ds.ds_layout_from_cuts([L] * b, [0, b])
            t[i, j] = runner.time_ms(lambda: runner.run(lay), reps=reps)
            if log:
                log("profile b=%d L=%d: %.3f ms" % (b, L, t[i, j]))
    return t


def build_table(b_grid, l_grid, t_ms, tb, tl):
    return ds.ds_cost_table_build(b_grid, l_grid, t_ms, tb, tl, scale=NS_PER_MS, inf_cost=INF_COST)


def micro_batch_layouts(layout, lens):
    """One single-micro-batch layout per micro-batch of `layout`, padded as in the plan, with its first row."""
    out = []
    order = lens[layout.perm]
    for m in range(layout.n_mb):
        s0, c = int(layout.mb_start[m]), int(layout.mb_count[m])
        sub = ds.ds_layout_from_cuts(order[s0:s0 + c], [0, c], pad_to=int(layout.mb_lpad[m]))
        out.append((sub, int(layout.mb_row[m])))
    return out


def measure_plan(runner, layout, lens, table, reps=3):
    """Predicted (table) against measured (one stage call per micro-batch, in plan order) times of a plan."""
    subs = micro_batch_layouts(layout, lens)
    tl = table.shape[1]
    pred_ns = np.array([table[int(layout.mb_count[m]) - 1, min(int(layout.mb_lpad[m]), tl) - 1] for m in range(layout.n_mb)],
                       dtype=np.float64)

    def sequential():
        for k, (sub, r0) in enumerate(subs):
            runner.run(sub, row0=r0, accumulate=k > 0)

    seq_ms = runner.time_ms(sequential, reps=reps)
    per_ms = np.array([runner.time_ms(lambda s=sub, r=r0: runner.run(s, row0=r), reps=reps) for sub, r0 in subs])
    grouped_ms = runner.time_ms(lambda: runner.run(layout), reps=reps)
    ok = pred_ns < INF_COST
    rel = np.abs(pred_ns[ok] / NS_PER_MS - per_ms[ok]) / per_ms[ok]
    return {
        "n_micro_batches": int(layout.n_mb),
        "rows": int(layout.total_rows),
        "padding_efficiency": float(layout.total_tokens) / float(layout.total_rows),
        "predicted_sum_ms": float(pred_ns[ok].sum() / NS_PER_MS),
        "predicted_max_ms": float(pred_ns[ok].max() / NS_PER_MS),
        "unpredicted_micro_batches": int((~ok).sum()),
        "measured_sequential_ms": seq_ms,
        "measured_sum_of_single_calls_ms": float(per_ms.sum()),
        "measured_max_single_call_ms": float(per_ms.max()),
        "measured_grouped_ms": grouped_ms,
        "per_micro_batch_mean_abs_rel_error": float(rel.mean()) if rel.size else None,
        "per_micro_batch_max_abs_rel_error": float(rel.max()) if rel.size else None,
        "sequential_prediction_rel_error": float(abs(pred_ns[ok].sum() / NS_PER_MS - seq_ms) / seq_ms),
    }


def report(config="gpt_2048_bf16", seed=0, reps=3, log=None):
    cfg = wl.CONFIGS[config]
    if cfg["kind"] != "gpt":
        raise SystemExit("the profiled cost model covers decoder-only stages")
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=seed)
    cap, c = cfg["cap"], cfg["num_stages"]
    lo, hi = cfg["lengths"]["lo"], cfg["lengths"]["hi"]
    tb = int(min(len(lens), cap // int(lens.min())))
    tl = int(lens.max())
    l_grid = power_of_two_grid(lo, tl)
    b_grid = power_of_two_grid(1, tb)
    poly = ds.dp_plan(lens, ds.make_cost_model(), cap, c)
    max_rows = int(max(poly.total_rows, 2 * cap))
    runner = StageRunner(cfg, max_rows=max_rows, max_seqs=max(len(lens), b_grid[-1]), seed=seed, same_weights=True)
    # profile up to twice the cap: every bracketing corner of an admissible (b, L) has b*L <= 4*cap, and the
    # interpolation marks cells whose corners were skipped as unaffordable only beyond b*L > cap
    t_ms = profile_grid(runner, b_grid, l_grid, max_rows=max_rows, reps=reps, log=log)
    table = build_table(b_grid, l_grid, t_ms, tb, tl)
    prof = ds.dp_plan(lens, ds.make_cost_model(kind=ds.DS_COST_TABLE, table=table), cap, c)
    tb_plans = {}
    for budget in (cap // 4, cap // 2, cap):        # the paper's TB baseline needs a search over its token budget
        tb_plans["plan_token_based_%d" % budget] = ds.ds_layout_token_based(lens, budget)
    need = max([int(prof.total_rows)] + [int(l.total_rows) for l in tb_plans.values()])
    if need > max_rows:                                 # plans that merge micro-batches pad: they need more rows
        runner.close()
        runner = StageRunner(cfg, max_rows=need, max_seqs=max(len(lens), b_grid[-1]), seed=seed, same_weights=True)
    out = {
        "config": config, "n_seq": int(len(lens)), "non_pad_tokens": int(lens.sum()), "cap": cap, "num_stages": c,
        "b_grid": b_grid, "l_grid": l_grid,
        "profile_ms": [[None if np.isnan(v) else round(float(v), 4) for v in row] for row in t_ms],
        "plan_polynomial_cost": measure_plan(runner, poly, lens, table, reps=reps),
        "plan_profiled_cost": measure_plan(runner, prof, lens, table, reps=reps),
    }
    for key, lay in tb_plans.items():
        out[key] = measure_plan(runner, lay, lens, table, reps=reps)
    for key in ["plan_polynomial_cost", "plan_profiled_cost"] + list(tb_plans):
        m = out[key]
        m["eq1_predicted_ms"] = (c - 1) * m["predicted_max_ms"] + m["predicted_sum_ms"]
        m["eq1_measured_ms"] = (c - 1) * m["measured_max_single_call_ms"] + m["measured_sum_of_single_calls_ms"]
    runner.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gpt_2048_bf16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    rep = report(args.config, args.seed, args.reps, log=lambda *a: print(*a, file=sys.stderr, flush=True))
    print(json.dumps(rep), flush=True)


if __name__ == "__main__":
    main()
