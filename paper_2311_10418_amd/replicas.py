"""Data-parallel replica balancing report (host only).

    python -m paper_2311_10418_amd.replicas --config gpt_2048_bf16 [--profile costmodel_report.json]

Plans the seeded batch for |D| = 1, 2, 4, 8 replicas with dp_plan_replicas (section "Micro-batch
Construction", paragraph "Balance data parallel model replicas") and prints, per |D|: planning time,
micro-batch count, the planner's lower bound  (c-1) max t + (1/|D|) sum t , the paper's upper bound of
the hybrid iteration time  (c-1) max t + max_d sum_d t  after the Karmarkar-Karp assignment, and the
imbalance max_d / mean_d.  With --profile (the JSON written by paper_2311_10418_amd.costmodel) the
profiled table cost is used instead of the polynomial one.  All arithmetic runs in the library.
"""
import argparse
import json
import time

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
    ds.lib()                                            # load the library outside the timed calls
    rows = []
    for D in (1, 2, 4, 8):
        t0 = time.perf_counter()
        lay, rep_of, sums = ds.dp_plan_replicas(lens, cm, cap, c, D, lengths_tgt=tgts)
        ms = (time.perf_counter() - t0) * 1e3
        lower = (c - 1) * int(lay.t_max) + int(sums.sum()) / D
        upper = (c - 1) * int(lay.t_max) + int(sums.max())
        rows.append({"replicas": D, "plan_ms": ms, "n_micro_batches": int(lay.n_mb),
                     "micro_batches_per_replica": [int((rep_of == r).sum()) for r in range(D)],
                     "lower_bound": lower, "upper_bound": upper, "upper_over_lower": upper / lower,
                     "imbalance_max_over_mean": float(sums.max() / (sums.sum() / D))})
    return {"config": config, "n_seq": int(len(lens)), "cost_unit": unit, "num_stages": c, "cap": cap, "plans": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gpt_2048_bf16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--profile", default=None)
    args = ap.parse_args()
    print(json.dumps(report(args.config, args.seed, args.profile)))


if __name__ == "__main__":
    main()
