"""Pipeline schedule report (host only).

    python -m paper_2311_10418_amd.schedule --config gpt_2048_bf16 [--profile costmodel_report.json]

Plans the seeded batch with dp_plan, gives every stage the same op times (forward 1/3, backward 2/3 of
the micro-batch's planned time t(M)) and activation sizes (padded rows), and compares, on the simulated
device timeline (section "Communication Planning"): the 1F1B order, the memory-aware adaptive schedule
(section "Pipeline Execution Schedule", Alg. 1) without a binding memory limit, and the adaptive
schedule limited to 1F1B's own peak memory.  Also prints Eq1's estimate (c-1) max t + sum t and the
length of the instruction streams of ds_comm_plan.  All arithmetic runs in the library.
"""
import argparse
import json

import numpy as np

from . import binding as ds
from . import workload as wl


def report(config, seed=0, profile=None):
    cfg = wl.CONFIGS[config]
    lens, tgts = wl.draw_lengths(cfg["lengths"], seed=seed)
    cap, c = cfg["cap"], cfg["num_stages"]
    if profile is not None:
        rep = json.load(open(profile))
        t = np.array([[np.nan if v is None else v for v in row] for row in rep["profile_ms"]], dtype=np.float64)
        tb = int(min(len(lens), cap // int(lens.min())))
        table = ds.ds_cost_table_build(rep["b_grid"], rep["l_grid"], t, tb, int(lens.max()), scale=1.0e6, inf_cost=1 << 50)
        cm, unit, tgts = ds.make_cost_model(kind=ds.DS_COST_TABLE, table=table), "ns (profiled table)", None
    elif cfg["kind"] == "t5":
        cm, unit = ds.make_cost_model(kind=ds.DS_COST_POLY_T5), "polynomial units"
    else:
        cm, unit, tgts = ds.make_cost_model(), "polynomial units", None
    lay = ds.dp_plan(lens, cm, cap, c, lengths_tgt=tgts)
    M = int(lay.n_mb)
    tm = lay.mb_cost.astype(np.int64)
    tf = np.repeat((tm // 3)[:, None], c, axis=1)
    tbw = np.repeat((tm - tm // 3)[:, None], c, axis=1)
    act = np.repeat((lay.mb_count.astype(np.int64) * lay.mb_lpad.astype(np.int64))[:, None], c, axis=1)
    out = {"config": config, "cost_unit": unit, "num_stages": c, "n_micro_batches": M,
           "eq1_estimate": int((c - 1) * tm.max() + tm.sum()), "sum_t": int(tm.sum()), "max_t": int(tm.max())}
    omb, okind = ds.ds_schedule_1f1b(c, M)
    s1 = ds.ds_schedule_simulate(omb, okind, tf, tbw, act)
    out["1f1b"] = {"makespan": int(s1["makespan"]), "peak_rows": s1["peak"].tolist(), "idle": s1["idle"].tolist()}
    for name, limit in (("adaptive_unlimited", np.full(c, act.sum() + 1)), ("adaptive_at_1f1b_peak", np.maximum(s1["peak"], act.max(axis=0)) + 1)):
        omb, okind, cycles = ds.ds_schedule_adaptive(act, limit)
        s = ds.ds_schedule_simulate(omb, okind, tf, tbw, act)
        stream = ds.ds_comm_plan(omb, okind, tf, tbw)
        out[name] = {"makespan": int(s["makespan"]), "vs_1f1b": float(s["makespan"]) / float(s1["makespan"]),
                     "peak_rows": s["peak"].tolist(), "cycles": cycles, "instructions_per_stage": [len(x) for x in stream]}
    out["eq1_over_1f1b"] = out["eq1_estimate"] / out["1f1b"]["makespan"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gpt_2048_bf16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--profile", default=None)
    args = ap.parse_args()
    print(json.dumps(report(args.config, args.seed, args.profile)))


if __name__ == "__main__":
    main()
