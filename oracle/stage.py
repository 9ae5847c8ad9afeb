"""TEST INFRASTRUCTURE: plain CPU oracle for one pipeline stage's forward and backward pass.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It shares no code with the product and never imports it.

What it computes.  The paper's executor runs, for every micro-batch, the
ForwardPass and BackwardPass instructions of one stage's transformer layers
(section "Overview", paragraph "Execution plans"), sums weight gradients over
the micro-batches of the iteration (section "Background", pipeline-parallel
paragraph) and claims the result equals ordinary padded or packed training
because samples are only regrouped inside a mini-batch (section "Related Work",
last sentence of the padding paragraph).  That equivalence is the plain
definition used here: every sequence is pushed through the layers ALONE and
UNPADDED, in float64, and weight gradients are summed over sequences.  No
micro-batch layout, padding or mask-for-padding exists in this file, which is
why layout independence and "pad positions contribute nothing" can be checked
against it.

Model definition where the paper is silent (it runs Megatron-LM's model code):
  GPT block, pre-LayerNorm:
      x1 = x  + Attn(LN1(x)) Wo + bo           causal, scale 1/sqrt(head_dim)
      x2 = x1 + GELU(LN2(x1) W1 + b1) W2 + b2  tanh-form GELU
      LayerNorm: biased variance, eps 1e-5, gain and bias.
  T5 block, pre-RMSNorm (gain only, eps 1e-6, no mean subtraction), no biases,
      gated-GELU MLP  (GELU(u Wg) * (u Wu)) W2.
      encoder layer: bidirectional self-attention, MLP.
      decoder layer: causal self-attention, cross-attention whose keys/values are
      the output of the stage's last encoder layer, MLP.
      scale 1/sqrt(head_dim), no relative-position bias.
Weights are stored [in_features, out_features]: y = x @ W.

parity pins (tests/test_oracle_stage.py): central finite differences of every
input and weight tensor, an autograd library's gradients of the same forward,
and closed-form special cases (single token, zero weights, constant rows, first
causal token).
"""
import math

import numpy as np

LN_EPS = 1e-5
RMS_EPS = 1e-6
_GELU_C = math.sqrt(2.0 / math.pi)
_GELU_A = 0.044715


# --------------------------------------------------------------------------- elementwise
def gelu(z):
    return 0.5 * z * (1.0 + np.tanh(_GELU_C * (z + _GELU_A * z ** 3)))


def gelu_grad(z):
    u = _GELU_C * (z + _GELU_A * z ** 3)
    t = np.tanh(u)
    du = _GELU_C * (1.0 + 3.0 * _GELU_A * z ** 2)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * du


# --------------------------------------------------------------------------- norms
def layernorm_fwd(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = xc * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, cache, g):
    xhat, rstd = cache
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def rmsnorm_fwd(x, g):
    ms = (x * x).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(ms + RMS_EPS)
    xhat = x * r
    return xhat * g, (xhat, r)


def rmsnorm_bwd(dy, cache, g):
    xhat, r = cache
    dg = (dy * xhat).sum(axis=0)
    dxhat = dy * g
    dx = r * (dxhat - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg


# --------------------------------------------------------------------------- attention
def attention_fwd(q, k, v, n_heads, causal):
    """q [lq, d], k/v [lk, d]; heads are consecutive column groups.  Returns o [lq, d] and a cache."""
    lq, d = q.shape
    lk = k.shape[0]
    hd = d // n_heads
    scale = 1.0 / math.sqrt(hd)
    o = np.zeros_like(q)
    probs = []
    for h in range(n_heads):
        cs = slice(h * hd, (h + 1) * hd)
        s = (q[:, cs] @ k[:, cs].T) * scale
        if causal:
            i = np.arange(lq)[:, None]
            j = np.arange(lk)[None, :]
            s = np.where(j <= i, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        e = np.exp(s)
        p = e / e.sum(axis=-1, keepdims=True)
        o[:, cs] = p @ v[:, cs]
        probs.append(p)
    return o, (q, k, v, probs, n_heads)


def attention_bwd(do, cache):
    q, k, v, probs, n_heads = cache
    d = q.shape[1]
    hd = d // n_heads
    scale = 1.0 / math.sqrt(hd)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(n_heads):
        cs = slice(h * hd, (h + 1) * hd)
        p = probs[h]
        dv[:, cs] = p.T @ do[:, cs]
        dp = do[:, cs] @ v[:, cs].T
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))     # softmax Jacobian, row-wise
        dq[:, cs] = (ds @ k[:, cs]) * scale
        dk[:, cs] = (ds.T @ q[:, cs]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------- GPT block
GPT_KEYS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def gpt_layer_fwd(x, p, n_heads):
    d = x.shape[1]
    u1, c_ln1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"])
    qkv = u1 @ p["w_qkv"] + p["b_qkv"]
    o, c_att = attention_fwd(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], n_heads, causal=True)
    x1 = x + o @ p["w_o"] + p["b_o"]
    u2, c_ln2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"])
    z = u2 @ p["w_1"] + p["b_1"]
    a = gelu(z)
    x2 = x1 + a @ p["w_2"] + p["b_2"]
    return x2, (c_ln1, u1, c_att, o, c_ln2, u2, z, a)


def gpt_layer_bwd(dx2, cache, p, g):
    """Adds this sequence's weight gradients into dict g; returns gradient of the layer input."""
    c_ln1, u1, c_att, o, c_ln2, u2, z, a = cache
    g["w_2"] += a.T @ dx2
    g["b_2"] += dx2.sum(axis=0)
    dz = (dx2 @ p["w_2"].T) * gelu_grad(z)
    g["w_1"] += u2.T @ dz
    g["b_1"] += dz.sum(axis=0)
    du2 = dz @ p["w_1"].T
    dx1_n, dg, db = layernorm_bwd(du2, c_ln2, p["ln2_g"])
    g["ln2_g"] += dg
    g["ln2_b"] += db
    dx1 = dx2 + dx1_n
    g["w_o"] += o.T @ dx1
    g["b_o"] += dx1.sum(axis=0)
    do = dx1 @ p["w_o"].T
    dq, dk, dv = attention_bwd(do, c_att)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    g["w_qkv"] += u1.T @ dqkv
    g["b_qkv"] += dqkv.sum(axis=0)
    du1 = dqkv @ p["w_qkv"].T
    dx_n, dg, db = layernorm_bwd(du1, c_ln1, p["ln1_g"])
    g["ln1_g"] += dg
    g["ln1_b"] += db
    return dx1 + dx_n


def _f64(params):
    return [{k: np.asarray(v, dtype=np.float64) for k, v in layer.items()} for layer in params]


def _zeros_like(params):
    return [{k: np.zeros_like(v) for k, v in layer.items()} for layer in params]


def gpt_stage_fwd(xs, params, n_heads):
    """Forward only: xs is a list of [l_i, d] arrays (one per sequence)."""
    params = _f64(params)
    outs = []
    for x in xs:
        h = np.asarray(x, dtype=np.float64)
        for p in params:
            h, _ = gpt_layer_fwd(h, p, n_heads)
        outs.append(h)
    return outs


def gpt_stage_fwd_bwd(xs, dys, params, n_heads):
    """xs, dys: lists of [l_i, d] arrays (stage input, upstream gradient of the stage output).

    Returns (outs, dxs, grads): per-sequence stage outputs, per-sequence gradients of the stage
    input, and weight gradients summed over all sequences (same structure as params).
    """
    params = _f64(params)
    grads = _zeros_like(params)
    outs, dxs = [], []
    for x, dy in zip(xs, dys):
        h = np.asarray(x, dtype=np.float64)
        caches = []
        for p in params:
            h, c = gpt_layer_fwd(h, p, n_heads)
            caches.append(c)
        outs.append(h)
        dh = np.asarray(dy, dtype=np.float64)
        for li in range(len(params) - 1, -1, -1):
            dh = gpt_layer_bwd(dh, caches[li], params[li], grads[li])
        dxs.append(dh)
    return outs, dxs, grads


# --------------------------------------------------------------------------- T5 blocks
T5_ENC_KEYS = ("ln1_g", "w_qkv", "w_o", "ln2_g", "w_g", "w_u", "w_2")
T5_DEC_KEYS = ("ln1_g", "w_qkv", "w_o", "lnc_g", "w_cq", "w_ckv", "w_co", "ln2_g", "w_g", "w_u", "w_2")


def _t5_mlp_fwd(x, p):
    u, c_ln = rmsnorm_fwd(x, p["ln2_g"])
    zg = u @ p["w_g"]
    zu = u @ p["w_u"]
    a = gelu(zg) * zu
    return x + a @ p["w_2"], (c_ln, u, zg, zu, a)


def _t5_mlp_bwd(dy, cache, p, g):
    c_ln, u, zg, zu, a = cache
    g["w_2"] += a.T @ dy
    da = dy @ p["w_2"].T
    dzg = da * zu * gelu_grad(zg)
    dzu = da * gelu(zg)
    g["w_g"] += u.T @ dzg
    g["w_u"] += u.T @ dzu
    du = dzg @ p["w_g"].T + dzu @ p["w_u"].T
    dx_n, dg = rmsnorm_bwd(du, c_ln, p["ln2_g"])
    g["ln2_g"] += dg
    return dy + dx_n


def _t5_self_fwd(x, p, n_heads, causal):
    d = x.shape[1]
    u, c_ln = rmsnorm_fwd(x, p["ln1_g"])
    qkv = u @ p["w_qkv"]
    o, c_att = attention_fwd(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], n_heads, causal)
    return x + o @ p["w_o"], (c_ln, u, c_att, o)


def _t5_self_bwd(dy, cache, p, g):
    c_ln, u, c_att, o = cache
    g["w_o"] += o.T @ dy
    do = dy @ p["w_o"].T
    dq, dk, dv = attention_bwd(do, c_att)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    g["w_qkv"] += u.T @ dqkv
    du = dqkv @ p["w_qkv"].T
    dx_n, dg = rmsnorm_bwd(du, c_ln, p["ln1_g"])
    g["ln1_g"] += dg
    return dy + dx_n


def _t5_cross_fwd(x, enc, p, n_heads):
    d = x.shape[1]
    u, c_ln = rmsnorm_fwd(x, p["lnc_g"])
    q = u @ p["w_cq"]
    kv = enc @ p["w_ckv"]
    o, c_att = attention_fwd(q, kv[:, :d], kv[:, d:], n_heads, causal=False)
    return x + o @ p["w_co"], (c_ln, u, c_att, o, enc)


def _t5_cross_bwd(dy, cache, p, g):
    """Returns (gradient of the decoder stream, gradient of the encoder output)."""
    c_ln, u, c_att, o, enc = cache
    g["w_co"] += o.T @ dy
    do = dy @ p["w_co"].T
    dq, dk, dv = attention_bwd(do, c_att)
    g["w_cq"] += u.T @ dq
    dkv = np.concatenate([dk, dv], axis=1)
    g["w_ckv"] += enc.T @ dkv
    denc = dkv @ p["w_ckv"].T
    du = dq @ p["w_cq"].T
    dx_n, dg = rmsnorm_bwd(du, c_ln, p["lnc_g"])
    g["lnc_g"] += dg
    return dy + dx_n, denc


def t5_stage_fwd_bwd(enc_xs, dec_xs, ddec_outs, enc_params, dec_params, n_heads):
    """Encoder-decoder stage.  Per sample: encoder input [l_in, d], decoder input [l_tgt, d],
    upstream gradient of the decoder output [l_tgt, d].

    Returns (dec_outs, d_enc_xs, d_dec_xs, enc_grads, dec_grads).
    """
    enc_params = _f64(enc_params)
    dec_params = _f64(dec_params)
    eg = _zeros_like(enc_params)
    dg_ = _zeros_like(dec_params)
    outs, d_enc, d_dec = [], [], []
    for ex, dx, ddy in zip(enc_xs, dec_xs, ddec_outs):
        e = np.asarray(ex, dtype=np.float64)
        enc_caches = []
        for p in enc_params:
            e, c1 = _t5_self_fwd(e, p, n_heads, causal=False)
            e, c2 = _t5_mlp_fwd(e, p)
            enc_caches.append((c1, c2))
        y = np.asarray(dx, dtype=np.float64)
        dec_caches = []
        for p in dec_params:
            y, c1 = _t5_self_fwd(y, p, n_heads, causal=True)
            y, c2 = _t5_cross_fwd(y, e, p, n_heads)
            y, c3 = _t5_mlp_fwd(y, p)
            dec_caches.append((c1, c2, c3))
        outs.append(y)
        dy = np.asarray(ddy, dtype=np.float64)
        de = np.zeros_like(e)
        for li in range(len(dec_params) - 1, -1, -1):
            c1, c2, c3 = dec_caches[li]
            dy = _t5_mlp_bwd(dy, c3, dec_params[li], dg_[li])
            dy, de_l = _t5_cross_bwd(dy, c2, dec_params[li], dg_[li])
            de += de_l
            dy = _t5_self_bwd(dy, c1, dec_params[li], dg_[li])
        d_dec.append(dy)
        for li in range(len(enc_params) - 1, -1, -1):
            c1, c2 = enc_caches[li]
            de = _t5_mlp_bwd(de, c2, enc_params[li], eg[li])
            de = _t5_self_bwd(de, c1, enc_params[li], eg[li])
        d_enc.append(de)
    return outs, d_enc, d_dec, eg, dg_
