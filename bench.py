#!/usr/bin/env python3
"""Benchmark: non-pad tokens/s of one stage's forward+backward over a DP-planned global batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--layout dp|fixed|packed]

One step = one stage_fwd_bwd call over the whole seeded synthetic global batch (every micro-batch
of the layout, forward and backward of every layer, weight gradients overwritten), inputs and
weights already resident in HBM.  Prints ONE JSON line on stdout; everything else goes to stderr.
The roofline figure is for the dominant kernel family (the bf16 MFMA GEMM), timed with HIP events
the library records on the launch stream inside the timed region.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_flops(cfg, lens, tgts=None):
    """Forward+backward flops the method must execute on non-pad tokens (causal half only)."""
    d, F, L = cfg["d_model"], cfg["d_ff"], cfg["n_layers"]
    tokens = int(lens.sum())
    if cfg["kind"] == "gpt":
        linear = 3 * 2 * (4 * d * d + 2 * d * F) * tokens * L
        attn = 3 * sum(2 * d * int(l) * (int(l) + 1) for l in lens) * L
        return linear, attn
    Ld = cfg["n_dec_layers"]
    ttok = int(tgts.sum())
    linear = 3 * (2 * (4 * d * d + 3 * d * F) * tokens * L + (2 * (6 * d * d + 3 * d * F) * ttok + 2 * 2 * d * d * tokens) * Ld)
    attn = 3 * (sum(4 * d * int(l) ** 2 for l in lens) * L +
                sum(2 * d * int(t) * (int(t) + 1) + 4 * d * int(t) * int(l) for l, t in zip(lens, tgts)) * Ld)
    return linear, attn


def build_layout(ds, kind, lens, cfg):
    if kind == "dp":
        return ds.dp_plan(lens, ds.make_cost_model(), cfg["cap"], cfg["num_stages"]), \
            "dp_plan c=%d cap=%d t=b*L*(1+L/2048)" % (cfg["num_stages"], cfg["cap"])
    hi = cfg["lengths"]["hi"]
    n = len(lens)
    if kind == "fixed":
        return ds.ds_layout_from_cuts(lens, list(range(0, n, 8)) + [n], pad_to=hi), "fixed padding to %d, 8 per micro-batch" % hi
    if kind == "packed":
        return ds.ds_layout_packed(lens, hi, 8), "first-fit packing into %d-token rows, 8 rows per micro-batch" % hi
    if kind == "packed_dense":
        # CONTEXT ONLY (timing, not the model's result): every packed row treated as ONE causal sequence, which is
        # the work a dense kernel with a block-diagonal mask does on packed input (section "Background", packing)
        pk = ds.ds_layout_packed(lens, hi, 8)
        fill = np.zeros(pk.total_rows // hi, dtype=np.int32)
        for r, l in zip(pk.seq_row, pk.seq_len):
            fill[r // hi] = max(fill[r // hi], r % hi + l)
        fill = fill[fill > 0]
        nrow = len(fill)
        return ds.ds_layout_from_cuts(fill, list(range(0, nrow, 8)) + [nrow], pad_to=hi), \
            "CONTEXT ONLY: packed rows attended densely (block-diagonal mask cost), %d-token rows, 8 per micro-batch" % hi
    raise SystemExit("unknown layout " + kind)


def cpu_baseline(cfg, lens, seed, budget_s=6.0):
    """The oracle, as it stands, on a bounded seeded sample of the same workload."""
    from oracle import stage as ost
    from paper_2311_10418_amd import workload as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    d, F, L = cfg["d_model"], cfg["d_ff"], cfg["n_layers"]
    n = 1024
    a = np.random.default_rng(0).standard_normal((n, n))
    t0 = time.perf_counter()
    a @ a
    rate = 2 * n ** 3 / (time.perf_counter() - t0)                      # fp64 flop/s of the host BLAS
    per_token = 3 * 2 * (4 * d * d + 2 * d * F) * L
    budget_tokens = int(min(max(budget_s * rate / per_token, 64), 8192))
    order = np.random.default_rng([seed, 9]).permutation(len(lens))
    pick, tok = [], 0
    for i in order:
        if tok + int(lens[i]) > budget_tokens and pick:
            continue
        pick.append(int(i))
        tok += int(lens[i])
        if tok >= budget_tokens:
            break
    params = wl.draw_params(wl.GPT_KEYS, L, d, F, seed=seed, bf16=True)
    params = [{k: v.astype(np.float64) for k, v in layer.items()} for layer in params]
    sub = lens[pick]
    xs = wl.draw_rows(sub, d, seed=seed, tag=3, bf16=True)
    dys = wl.draw_rows(sub, d, seed=seed, tag=5, bf16=True)
    t0 = time.perf_counter()
    ost.gpt_stage_fwd_bwd(xs, dys, params, cfg["n_heads"])
    dt = time.perf_counter() - t0
    return {"value": tok / dt, "unit": "non-pad tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d seeded sequences of the batch, %d tokens, float64 numpy, %.1f s" % (len(pick), tok, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="gpt_2048_bf16")
    ap.add_argument("--layout", default="dp", choices=["dp", "fixed", "packed", "packed_dense"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--recompute", default="none", choices=["none", "full"],
                    help="full: keep only layer inputs and re-run each layer's forward before its backward (context; "
                         "the headline keeps every activation)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    import torch
    from paper_2311_10418_amd import binding as ds
    from paper_2311_10418_amd import workload as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    cfg = wl.CONFIGS[args.config]
    t5 = cfg["kind"] == "t5"
    recompute = ds.DS_RECOMPUTE_FULL if args.recompute == "full" else ds.DS_RECOMPUTE_NONE
    dev = "cuda:0"
    torch.cuda.set_device(0)
    lens, tgts = wl.draw_lengths(cfg["lengths"], seed=args.seed)
    t0 = time.perf_counter()
    if t5:
        if args.layout != "dp":
            raise SystemExit("only the DP-planned layout is timed for the encoder-decoder stage")
        layout = ds.dp_plan(lens, ds.make_cost_model(kind=ds.DS_COST_POLY_T5), cfg["cap"], cfg["num_stages"], lengths_tgt=tgts)
        layout_desc = "dp_plan c=%d cap=%d encoder-decoder cost" % (cfg["num_stages"], cfg["cap"])
    else:
        layout, layout_desc = build_layout(ds, args.layout, lens, cfg)
    plan_ms = (time.perf_counter() - t0) * 1e3
    d, F, L, H = cfg["d_model"], cfg["d_ff"], cfg["n_layers"], cfg["n_heads"]
    bf16 = cfg["dtype"] == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    code = ds.DS_DTYPE_BF16 if bf16 else ds.DS_DTYPE_F32
    R = layout.total_rows
    log("workload %s: %d sequences, %d non-pad tokens, %d rows in %d micro-batches (%s), plan %.2f ms"
        % (args.config, len(lens), layout.total_tokens, R, layout.n_mb, layout_desc, plan_ms))

    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    shapes = {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (d, 3 * d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
              "ln2_g": (d,), "ln2_b": (d,), "w_1": (d, F), "b_1": (F,), "w_2": (F, d), "b_2": (d,),
              "lnc_g": (d,), "w_g": (d, F), "w_u": (d, F), "w_cq": (d, d), "w_ckv": (d, 2 * d), "w_co": (d, d)}

    def make_layers(keys, n):
        ws, gs = [], []
        for _ in range(n):
            w, g = {}, {}
            for k in keys:
                v = torch.randn(shapes[k], generator=gen, device=dev, dtype=torch.float32) * 0.02
                if k.endswith("_g") and k.startswith("ln"):
                    v = v + 1.0
                w[k] = v.to(tdt).contiguous()
                g[k] = torch.zeros(shapes[k], device=dev, dtype=torch.float32)
            ws.append(w)
            gs.append(g)
        return ws, gs

    def rnd(rows):
        return torch.randn((rows, d), generator=gen, device=dev, dtype=torch.float32).to(tdt)

    if t5:
        Rt = layout.total_rows_tgt
        weights, grads = make_layers(ds.T5_ENC_KEYS, L)
        weights_d, grads_d = make_layers(ds.T5_DEC_KEYS, cfg["n_dec_layers"])
        x, y, dy = rnd(R), rnd(Rt), rnd(Rt)
        out, dx, dyin = torch.empty_like(y), torch.empty_like(x), torch.empty_like(y)
        stage = ds.Stage(ds.DS_MODEL_T5, code, L, d, H, F, max_rows=R, max_seqs=len(lens),
                         n_dec_layers=cfg["n_dec_layers"], max_rows_tgt=Rt, recompute=recompute)

        def step():
            ds.stage_fwd_bwd(stage, layout, weights, x, dy, out, dx, grads, accumulate=False, weights_dec=weights_d,
                             grads_dec=grads_d, act_in_tgt=y, grad_in_tgt=dyin)
    else:
        weights, grads = make_layers(ds.GPT_KEYS, L)
        x, dy = rnd(R), rnd(R)
        out, dx = torch.empty_like(x), torch.empty_like(x)
        stage = ds.Stage(ds.DS_MODEL_GPT, code, L, d, H, F, max_rows=R, max_seqs=max(len(lens), layout.n_seq),
                         recompute=recompute)

        def step():
            ds.stage_fwd_bwd(stage, layout, weights, x, dy, out, dx, grads, accumulate=False)
    workspace_gb = stage.workspace_bytes() / 2 ** 30
    log("workspace %.2f GB" % workspace_gb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stage.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = stage.profile_read()
    stage.profile_enable(False)
    ms_per_step = elapsed * 1e3 / args.steps
    tokens = int(layout.total_tokens) + int(layout.total_tokens_tgt)
    value = tokens / (elapsed / args.steps)

    lin_flops, attn_flops = algorithmic_flops(cfg, lens, tgts)
    gemm_ms = sum(prof[k][0] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad")) / args.steps
    gemm_launches = sum(prof[k][1] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad")) // args.steps
    achieved = lin_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    breakdown = {k: round(v[0] / args.steps, 4) for k, v in prof.items()}
    log("per-step ms by kernel group:", json.dumps(breakdown))
    log("launches per step: %d" % stage.last_launch_count())
    useful_util = (lin_flops + attn_flops) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
    all_rows = R + int(layout.total_rows_tgt)
    log("useful MFMA utilisation (all algorithmic flops / step time / %.0f TFLOP/s): %.4f" % (PEAK_BF16_TFLOPS, useful_util))
    log("padding efficiency %.4f" % (tokens / all_rows))

    # HBM-side bytes per GEMM launch from the committed rocprofv3 --pmc summary of this same command, if it
    # covers this workload (FETCH_SIZE / WRITE_SIZE scaled by a plain copy of known size); else null.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_traffic_%s.json" % args.config)
    if args.layout == "dp" and os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")

    result = {
        "metric": "non-pad tokens/s, stage fwd+bwd bf16 on 1 MI355X; MFMA util % of peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "mfma_util_pct_of_peak": 100.0 * useful_util,      # second part of the metric: useful flops of the whole step
        "config": {"workload": args.config, "stage_shape": "%d layers d_model %d heads %d d_ff %d" % (L, d, H, F),
                   "layout": layout_desc, "n_seq": int(len(lens)), "non_pad_tokens": tokens, "rows": int(all_rows),
                   "n_micro_batches": int(layout.n_mb), "padding_efficiency": tokens / all_rows,
                   "dp_plan_ms": plan_ms, "recompute": args.recompute, "workspace_gb": round(workspace_gb, 3),
                   "useful_mfma_utilisation": useful_util,
                   "ms_per_step_by_group": breakdown},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_nt_kernel (all projections: forward, dgrad, wgrad)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "launches_per_step": int(gemm_launches), "ms_per_step": gemm_ms,
                     "algorithmic_flops_per_step": lin_flops},
    }
    # One plain device copy of known size (256 MiB read + 256 MiB written), outside the timed region: the
    # reference dispatch against which FETCH_SIZE / WRITE_SIZE counters of a profiler run are scaled.
    cal_src = torch.ones(64 * 2 ** 20, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    stage.close()
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and not t5:
        result["cpu_baseline"] = cpu_baseline(cfg, lens, args.seed)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
