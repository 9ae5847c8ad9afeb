"""Shared plumbing for the GPU parity tests: move seeded inputs to the device in a layout's stream
order, run the HIP path through the C ABI, bring results back per sequence, compare with the
oracle.  No method arithmetic here."""
import numpy as np
import torch

from paper_2311_10418_amd import binding as ds

DEV = "cuda:0"


def tdtype(code):
    return torch.bfloat16 if code == ds.DS_DTYPE_BF16 else torch.float32


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return num / den if den > 0 else num


MAX_FACTOR = 8.0       # elementwise companion of a normwise bound tol: |got - ref| <= tol * (MAX_FACTOR * rms(ref) + |ref|)


def max_err(got, ref):
    """Largest elementwise deviation in units of MAX_FACTOR * rms(ref) + |ref| (the root mean square of the whole
    reference tensor sets the absolute scale; the |ref| term lets an element far in the tail of a heavy-tailed
    tensor carry the rounding error of its own magnitude)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref.ravel() ** 2))
    den = MAX_FACTOR * rms + np.abs(ref)
    dev = np.abs(got - ref)
    if rms == 0:
        return float(dev.max())
    return float((dev / den).max())


def both_err(got, ref):
    """max(normwise relative error, elementwise error in the units of max_err): `both_err(...) <= tol` asserts the
    normwise bound and its elementwise companion at once."""
    return max(rel_err(got, ref), max_err(got, ref))


def check(got, ref, tol, tag=""):
    """One tensor against the oracle: normwise relative error <= tol AND every element within
    tol * (MAX_FACTOR * rms(ref) + |ref|) (a wrong column slice, row or tile cannot hide inside the norm of a large
    tensor).  Returns the normwise error."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (tag, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), (tag, "non-finite values")
    e, m = rel_err(got, ref), max_err(got, ref)
    assert e <= tol, (tag, "normwise", e, tol)
    assert m <= tol, (tag, "elementwise", m, tol)
    return e


def check_seqs(got_seqs, ref_seqs, tol, tag=""):
    """Per-sequence tensors (outputs, input gradients): every sequence on its own meets the bound."""
    assert len(got_seqs) == len(ref_seqs), tag
    worst = 0.0
    for i, (g, r) in enumerate(zip(got_seqs, ref_seqs)):
        worst = max(worst, check(g, r, tol, "%s seq %d len %d" % (tag, i, np.asarray(r).shape[0])))
    return worst


def to_dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dtype).contiguous()


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def stream_from_seqs(seqs, layout, d, dtype, fill=float("nan"), which=0):
    """seqs: per-sequence [l_i, d] arrays in ORIGINAL order -> [total_rows, d] device tensor, pad rows = fill."""
    rows = layout.total_rows_tgt if which else layout.total_rows
    seq_row = layout.seq_row_tgt if which else layout.seq_row
    host = np.full((rows, d), fill, dtype=np.float32)
    for s in range(layout.n_seq):
        a = seqs[int(layout.perm[s])]
        host[seq_row[s]:seq_row[s] + a.shape[0]] = a
    return torch.from_numpy(host).to(DEV).to(dtype).contiguous()


def seqs_from_stream(t, layout, which=0):
    """-> (per-sequence arrays in ORIGINAL order, array of all padding rows)."""
    host = to_np(t)
    seq_row = layout.seq_row_tgt if which else layout.seq_row
    seq_len = layout.seq_len_tgt if which else layout.seq_len
    out = [None] * layout.n_seq
    mask = np.ones(host.shape[0], dtype=bool)
    for s in range(layout.n_seq):
        r, l = int(seq_row[s]), int(seq_len[s])
        out[int(layout.perm[s])] = host[r:r + l]
        mask[r:r + l] = False
    return out, host[mask]


def params_to_dev(params, dtype):
    return [{k: to_dev(v, dtype) for k, v in layer.items()} for layer in params]


def zero_grads_like(params_dev):
    return [{k: torch.zeros(v.shape, dtype=torch.float32, device=DEV) for k, v in layer.items()} for layer in params_dev]


def run_gpt_stage(layout, cfg, params, xs, dys, dtype_code, stage=None, fill=float("nan"), accumulate=False, grads=None,
                  recompute=0):
    """Run stage_fwd_bwd on a layout.  Returns (outs, dxs, grads_np, pad_out_rows, pad_dx_rows)."""
    dt = tdtype(dtype_code)
    d = cfg["d_model"]
    own = stage is None
    if own:
        stage = ds.Stage(ds.DS_MODEL_GPT, dtype_code, cfg["n_layers"], d, cfg["n_heads"], cfg["d_ff"],
                         max_rows=layout.total_rows, max_seqs=layout.n_seq, recompute=recompute)
    w = params_to_dev(params, dt)
    if grads is None:
        grads = zero_grads_like(w)
    x = stream_from_seqs(xs, layout, d, dt, fill)
    dy = stream_from_seqs(dys, layout, d, dt, fill)
    out = torch.full_like(x, 7.0)
    dx = torch.full_like(x, 7.0)
    ds.stage_fwd_bwd(stage, layout, w, x, dy, out, dx, grads, accumulate=accumulate)
    torch.cuda.synchronize()
    outs, pad_o = seqs_from_stream(out, layout)
    dxs, pad_dx = seqs_from_stream(dx, layout)
    g_np = [{k: to_np(v) for k, v in layer.items()} for layer in grads]
    if own:
        stage.close()
    return outs, dxs, g_np, pad_o, pad_dx


def cat(seqs):
    return np.concatenate([np.asarray(s, dtype=np.float64) for s in seqs], axis=0)


def run_t5_stage(layout, cfg, enc_params, dec_params, enc_xs, dec_xs, ddec, dtype_code, fill=float("nan"), recompute=0):
    """Encoder-decoder stage on a two-stream layout.  Returns dict of per-sequence outputs / gradients,
    weight gradients (numpy) and the padding rows of every output stream."""
    dt = tdtype(dtype_code)
    d = cfg["d_model"]
    stage = ds.Stage(ds.DS_MODEL_T5, dtype_code, cfg["n_layers"], d, cfg["n_heads"], cfg["d_ff"],
                     max_rows=layout.total_rows, max_seqs=layout.n_seq, n_dec_layers=cfg["n_dec_layers"],
                     max_rows_tgt=layout.total_rows_tgt, recompute=recompute)
    we, wd = params_to_dev(enc_params, dt), params_to_dev(dec_params, dt)
    ge, gd = zero_grads_like(we), zero_grads_like(wd)
    x = stream_from_seqs(enc_xs, layout, d, dt, fill, which=0)
    y = stream_from_seqs(dec_xs, layout, d, dt, fill, which=1)
    dy = stream_from_seqs(ddec, layout, d, dt, fill, which=1)
    out = torch.full_like(y, 7.0)
    dx = torch.full_like(x, 7.0)
    dyin = torch.full_like(y, 7.0)
    ds.stage_fwd_bwd(stage, layout, we, x, dy, out, dx, ge, weights_dec=wd, grads_dec=gd, act_in_tgt=y, grad_in_tgt=dyin)
    torch.cuda.synchronize()
    outs, pad_o = seqs_from_stream(out, layout, which=1)
    d_enc, pad_e = seqs_from_stream(dx, layout, which=0)
    d_dec, pad_d = seqs_from_stream(dyin, layout, which=1)
    res = {"outs": outs, "d_enc": d_enc, "d_dec": d_dec,
           "eg": [{k: to_np(v) for k, v in layer.items()} for layer in ge],
           "dg": [{k: to_np(v) for k, v in layer.items()} for layer in gd],
           "pads": [pad_o, pad_e, pad_d]}
    stage.close()
    return res
