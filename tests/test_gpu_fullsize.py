"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (DP plan of the
whole seeded global batch, full model), and on the fixed-padding and packed layouts of the same batch.
The oracle cannot run 65 K tokens through a 200 M-parameter stage in test time, so:
  * stage outputs and input gradients are per-sequence independent, hence checked against the oracle
    on SAMPLED sequences (their rows come from the seeded generator, all other rows are device noise,
    padding rows are NaN); the sample always holds the shortest, a median, a mid-length and the LONGEST
    sequence of the batch (the longest one sits in the last rows of the stream, where row x d_ff passes
    2^31 elements at the long-tail configuration);
  * weight gradients are sums over sequences: the oracle checks them (a) on the sampled sub-batch run
    through the full-size model, (b) directly on a 16 K-token batch through one full-width layer, where
    the contraction over tokens is split over whole rounds of work-groups as at full size, and
    (c) additivity over disjoint halves of the batch ties the full-batch gradients to sub-batch ones.
Every comparison is normwise (2e-2, bf16) per sequence / per tensor plus the elementwise companion bound
of helpers.check.
"""
import numpy as np
import pytest
import torch

from oracle import stage as ost
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl
from helpers import DEV, check, params_to_dev, rel_err, to_np, zero_grads_like

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _rows_for(lens, idx, d, seed, tag):
    """Seeded rows of one original-order sequence (same values draw_rows gives it)."""
    rng = np.random.default_rng([seed, tag, int(idx)])
    return wl.to_bf16_grid(rng.standard_normal((int(lens[idx]), d), dtype=np.float32))


def _run(stage, layout, w, x, dy):
    out = torch.full_like(x, 7.0)
    dx = torch.full_like(x, 7.0)
    g = zero_grads_like(w)
    ds.stage_fwd_bwd(stage, layout, w, x, dy, out, dx, g)
    torch.cuda.synchronize()
    return out, dx, g


def _oracle_by_sequence(xs, dys, params, n_heads, tag):
    """The oracle one sequence at a time (it treats sequences independently and sums their weight gradients, so this
    is its own definition spelt out), with a progress line after each: a long run stays visibly alive."""
    import time
    outs, dxs, grads = [], [], None
    for j, (x, dy) in enumerate(zip(xs, dys)):
        t0 = time.time()
        o, g, w = ost.gpt_stage_fwd_bwd([x], [dy], params, n_heads)
        outs.append(o[0])
        dxs.append(g[0])
        if grads is None:
            grads = w
        else:
            for li, layer in enumerate(w):
                for k, v in layer.items():
                    grads[li][k] = grads[li][k] + v
        print("  oracle %s: sequence %d of %d, %d tokens, %.1f s" % (tag, j + 1, len(xs), x.shape[0], time.time() - t0), flush=True)
    return outs, dxs, grads


def _sample(lens, sample_tokens, long_len):
    """Shortest, median, one near long_len, the longest, then mid-length ones up to the token budget."""
    order = np.argsort(lens, kind="stable")
    pick = [int(order[0]), int(order[len(order) // 2]), int(np.argmin(np.abs(lens.astype(np.int64) - long_len))),
            int(order[-1])]
    pick = list(dict.fromkeys(pick))
    budget = sample_tokens + int(lens[pick].sum())
    tok = int(lens[pick].sum())
    for i in order[len(order) // 2 + 1:]:
        if int(i) in pick:
            continue
        if tok + int(lens[i]) > budget:
            break
        pick.append(int(i))
        tok += int(lens[i])
    return pick


def _noise_stream(layout, d, gen):
    """[rows, d] device noise in the rows of sequences, NaN in every padding row."""
    R = layout.total_rows
    x = torch.randn((R, d), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    if layout.total_rows != layout.total_tokens:
        valid = torch.zeros(R, dtype=torch.bool)
        for s in range(layout.n_seq):
            valid[int(layout.seq_row[s]):int(layout.seq_row[s]) + int(layout.seq_len[s])] = True
        x[~valid.to(DEV)] = float("nan")
    return x


def _pad_rows_zero(t, layout):
    R = layout.total_rows
    valid = torch.zeros(R, dtype=torch.bool)
    for s in range(layout.n_seq):
        valid[int(layout.seq_row[s]):int(layout.seq_row[s]) + int(layout.seq_len[s])] = True
    pad = t[~valid.to(DEV)]
    return pad.numel() == 0 or bool((pad == 0).all().item())


def _layouts_for(name, lens, cfg):
    yield "dp", ds.dp_plan(lens, ds.make_cost_model(), cfg["cap"], cfg["num_stages"])
    if name == "gpt_2048_bf16":
        # the layout comparison of the same seeded batch: first-fit packing and fixed padding, 8 rows per micro-batch
        hi, n = cfg["lengths"]["hi"], len(lens)
        yield "packed", ds.ds_layout_packed(lens, hi, 8)
        yield "fixed", ds.ds_layout_from_cuts(lens, list(range(0, n, 8)) + [n], pad_to=hi)


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("name,sample_tokens,long_len", [("gpt_2048_bf16", 700, 1100), ("gpt_4096_longtail_bf16", 350, 700)])
def test_full_size_configuration(name, sample_tokens, long_len):
    cfg = wl.CONFIGS[name]
    d, F, L, H = cfg["d_model"], cfg["d_ff"], cfg["n_layers"], cfg["n_heads"]
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=0)
    params = wl.draw_params(wl.GPT_KEYS, L, d, F, seed=0, bf16=True)
    w = params_to_dev(params, torch.bfloat16)
    pick = _sample(lens, sample_tokens, long_len)
    assert int(lens[pick].max()) == int(lens.max())
    print(name, "sampled sequences", pick, "lengths", [int(lens[i]) for i in pick], flush=True)
    xs = [_rows_for(lens, i, d, 0, 3) for i in pick]
    dys = [_rows_for(lens, i, d, 0, 5) for i in pick]
    r_outs, r_dxs, r_grads = _oracle_by_sequence(xs, dys, params, H, name)

    for lname, layout in _layouts_for(name, lens, cfg):
        R = layout.total_rows
        if lname == "dp":
            assert layout.total_rows == layout.total_tokens == int(lens.sum())
        else:
            assert layout.total_rows > layout.total_tokens
        gen = torch.Generator(device=DEV)
        gen.manual_seed(1)
        x, dy = _noise_stream(layout, d, gen), _noise_stream(layout, d, gen)
        pos_of = {int(layout.perm[s]): s for s in range(layout.n_seq)}
        for j, i in enumerate(pick):
            r0 = int(layout.seq_row[pos_of[i]])
            x[r0:r0 + xs[j].shape[0]] = torch.from_numpy(xs[j]).to(DEV).to(torch.bfloat16)
            dy[r0:r0 + xs[j].shape[0]] = torch.from_numpy(dys[j]).to(DEV).to(torch.bfloat16)
        stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, L, d, H, F, max_rows=R, max_seqs=len(lens))
        out, dx, g_full = _run(stage, layout, w, x, dy)

        # 1. sampled sequences against the oracle; padding rows exactly zero
        for j, i in enumerate(pick):
            r0, l = int(layout.seq_row[pos_of[i]]), int(lens[i])
            e_o = check(to_np(out[r0:r0 + l]), r_outs[j], TOL, "%s %s seq %d act_out" % (name, lname, i))
            e_g = check(to_np(dx[r0:r0 + l]), r_dxs[j], TOL, "%s %s seq %d grad_in" % (name, lname, i))
            print("  %s seq %d len %d first row %d: act_out %.2e grad_in %.2e" % (lname, i, l, r0, e_o, e_g), flush=True)
        assert _pad_rows_zero(out, layout) and _pad_rows_zero(dx, layout), lname
        for li in range(L):
            for k, v in g_full[li].items():
                assert bool(torch.isfinite(v).all().item()), (lname, li, k)
        if lname != "dp":
            stage.close()
            del out, dx, g_full, x, dy
            torch.cuda.empty_cache()
            continue

        # 2. the sampled sub-batch through the full-size model: weight gradients against the oracle
        sub_lens = lens[pick]
        lo_sub = ds.dp_plan(sub_lens, ds.make_cost_model(), cfg["cap"], cfg["num_stages"])
        xsub = torch.cat([torch.from_numpy(xs[int(lo_sub.perm[s])]) for s in range(lo_sub.n_seq)]).to(DEV).to(torch.bfloat16)
        dysub = torch.cat([torch.from_numpy(dys[int(lo_sub.perm[s])]) for s in range(lo_sub.n_seq)]).to(DEV).to(torch.bfloat16)
        _, _, g_sub = _run(stage, lo_sub, w, xsub.contiguous(), dysub.contiguous())
        worst = 0.0
        for li in range(L):
            for k, v in r_grads[li].items():
                worst = max(worst, check(to_np(g_sub[li][k]), v, TOL, "%s sub-batch L%d.%s" % (name, li, k)))
        print("  sub-batch weight gradients, worst %.2e" % worst, flush=True)

        # 3. additivity over disjoint halves of the batch (even / odd sorted positions)
        halves = []
        for par in (0, 1):
            pos = [s for s in range(layout.n_seq) if s % 2 == par]
            rows = torch.cat([torch.arange(int(layout.seq_row[s]), int(layout.seq_row[s]) + int(layout.seq_len[s])) for s in pos]).to(DEV)
            hl = np.array([int(layout.seq_len[s]) for s in pos], dtype=np.int32)
            lo_h = ds.ds_layout_from_cuts(hl, list(range(len(hl) + 1)))          # already sorted: one sequence per micro-batch
            _, _, g_h = _run(stage, lo_h, w, x.index_select(0, rows).contiguous(), dy.index_select(0, rows).contiguous())
            halves.append(g_h)
        worst = 0.0
        for li in range(L):
            for k in g_full[li]:
                ref = to_np(g_full[li][k])
                e = rel_err(to_np(halves[0][li][k]) + to_np(halves[1][li][k]), ref)
                worst = max(worst, e)
                assert e <= 2e-3, (li, k, e)
        print("  additivity of weight gradients over halves, worst %.2e" % worst, flush=True)
        stage.close()
        del out, dx, g_full, x, dy, halves
        torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_full_width_weight_gradients_over_16k_tokens_against_the_oracle():
    """One layer of the gpt_2048_bf16 model over the first sequences of its seeded batch that hold at least 16384
    tokens: EVERY weight-gradient tensor (and every sequence's output and input gradient) against the oracle
    directly.  The token contraction of the weight-gradient GEMMs (K = 16 K rows) is then split over whole rounds
    of work-groups and summed by the finishing kernel, the path the full-size batch takes."""
    cfg = wl.CONFIGS["gpt_2048_bf16"]
    d, F, H = cfg["d_model"], cfg["d_ff"], cfg["n_heads"]
    lens_all, _ = wl.draw_lengths(cfg["lengths"], seed=0)
    n = int(np.searchsorted(np.cumsum(lens_all), 16384)) + 1
    lens = lens_all[:n]
    assert int(lens.sum()) >= 16384
    params = wl.draw_params(wl.GPT_KEYS, 1, d, F, seed=0, bf16=True)
    xs = wl.draw_rows(lens, d, seed=0, tag=3, bf16=True)
    dys = wl.draw_rows(lens, d, seed=0, tag=5, bf16=True)
    print("16k case: %d sequences, %d tokens, longest %d" % (n, int(lens.sum()), int(lens.max())), flush=True)
    from helpers import check_seqs, run_gpt_stage
    layout = ds.dp_plan(lens, ds.make_cost_model(), cfg["cap"], cfg["num_stages"])
    outs, dxs, grads, _, _ = run_gpt_stage(layout, dict(cfg, n_layers=1), params, xs, dys, ds.DS_DTYPE_BF16)
    r_outs, r_dxs, r_grads = _oracle_by_sequence(xs, dys, params, H, "16k")
    check_seqs(outs, r_outs, TOL, "16k act_out")
    check_seqs(dxs, r_dxs, TOL, "16k grad_in")
    for k, v in r_grads[0].items():
        e = check(grads[0][k], v, TOL, "16k " + k)
        print("  %-6s %.2e" % (k, e), flush=True)


@pytest.mark.timeout(900)
def test_full_size_encoder_decoder_configuration():
    """t5_1024_bf16 at its full size (DP plan of the whole seeded batch, 2 + 2 layers, d = 1024, head dimension 64):
    decoder outputs and both input gradients of SAMPLED samples against the oracle (samples are independent of each
    other), weight gradients on the sampled sub-batch."""
    from helpers import run_t5_stage
    name = "t5_1024_bf16"
    cfg = wl.CONFIGS[name]
    d, F, H = cfg["d_model"], cfg["d_ff"], cfg["n_heads"]
    lens, tgts = wl.draw_lengths(cfg["lengths"], seed=0)
    cm = ds.make_cost_model(kind=ds.DS_COST_POLY_T5)
    layout = ds.dp_plan(lens, cm, cfg["cap"], cfg["num_stages"], lengths_tgt=tgts)
    ep = wl.draw_params(wl.T5_ENC_KEYS, cfg["n_layers"], d, F, seed=0, tag=6, bf16=True)
    dp = wl.draw_params(wl.T5_DEC_KEYS, cfg["n_dec_layers"], d, F, seed=0, tag=7, bf16=True)
    ex = wl.draw_rows(lens, d, seed=0, tag=3, bf16=True)
    dx = wl.draw_rows(tgts, d, seed=0, tag=8, bf16=True)
    ddy = wl.draw_rows(tgts, d, seed=0, tag=5, bf16=True)
    # sampled samples: shortest and longest input, one near 700, longest target, and median ones up to a token budget
    order = np.argsort(lens, kind="stable")
    pick = {int(order[0]), int(order[-1]), int(np.argmin(np.abs(lens.astype(np.int64) - 700))), int(np.argmax(tgts))}
    budget = int(sum(lens[i] for i in pick)) + 1100
    tok = int(sum(lens[i] for i in pick))
    for i in order[len(order) // 2:]:
        if tok + int(lens[i]) > budget:
            break
        if int(i) not in pick:
            pick.add(int(i))
            tok += int(lens[i])
    pick = sorted(pick)
    print(name, "sampled", pick, "input lengths", [int(lens[i]) for i in pick], "target lengths", [int(tgts[i]) for i in pick], flush=True)

    got = run_t5_stage(layout, cfg, ep, dp, ex, dx, ddy, ds.DS_DTYPE_BF16)
    sub = lambda seqs: [seqs[i] for i in pick]
    r_outs, r_denc, r_ddec, r_eg, r_dg = ost.t5_stage_fwd_bwd(sub(ex), sub(dx), sub(ddy), ep, dp, H)
    for j, i in enumerate(pick):
        e = (check(got["outs"][i], r_outs[j], TOL, "t5 sample %d dec_out" % i),
             check(got["d_enc"][i], r_denc[j], TOL, "t5 sample %d d_enc_in" % i),
             check(got["d_dec"][i], r_ddec[j], TOL, "t5 sample %d d_dec_in" % i))
        print("  sample", i, "dec_out %.2e d_enc_in %.2e d_dec_in %.2e" % e, flush=True)
    for p in got["pads"]:
        assert p.size == 0 or np.all(p == 0)

    # the sampled sub-batch through the full-size model: weight gradients against the oracle
    sl, st_ = lens[pick], tgts[pick]
    lo_sub = ds.dp_plan(sl, cm, cfg["cap"], cfg["num_stages"], lengths_tgt=st_)
    got_sub = run_t5_stage(lo_sub, cfg, ep, dp, sub(ex), sub(dx), sub(ddy), ds.DS_DTYPE_BF16)
    worst = 0.0
    for tag, gg, rr in (("enc", got_sub["eg"], r_eg), ("dec", got_sub["dg"], r_dg)):
        for li, layer in enumerate(rr):
            for k, v in layer.items():
                worst = max(worst, check(gg[li][k], v, TOL, "t5 sub-batch %s%d.%s" % (tag, li, k)))
    print("  sub-batch weight gradients, worst %.2e" % worst, flush=True)
