"""Pins for the stage oracle (oracle/stage.py).  Nothing here calls the product.

  - central finite differences in float64 on tiny shapes, for every input and weight tensor;
  - the gradients an autograd library derives from its own forward of the same model;
  - closed forms: one-token sequences, zero projection weights, constant rows, first causal token;
  - per-sequence independence: results of a sequence do not depend on what else is in the batch.
"""
import math

import numpy as np
import pytest
import torch

from oracle import stage as ost


def _rand_params(keys, n_layers, d, f, rng, std=0.3):
    shape = {"ln1_g": (d,), "ln1_b": (d,), "ln2_g": (d,), "ln2_b": (d,), "lnc_g": (d,),
             "w_qkv": (d, 3 * d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
             "w_1": (d, f), "b_1": (f,), "w_2": (f, d), "b_2": (d,), "w_g": (d, f), "w_u": (d, f),
             "w_cq": (d, d), "w_ckv": (d, 2 * d), "w_co": (d, d)}
    out = []
    for _ in range(n_layers):
        layer = {}
        for k in keys:
            v = rng.standard_normal(shape[k]) * std
            if k.startswith("ln") and k.endswith("_g"):
                v = 1.0 + v
            layer[k] = v
        out.append(layer)
    return out


def _gpt_loss(xs, dys, params, h):
    outs = ost.gpt_stage_fwd(xs, params, h)
    return sum(float((o * dy).sum()) for o, dy in zip(outs, dys))


def test_gpt_finite_differences():
    rng = np.random.default_rng(0)
    d, h, f = 8, 2, 12
    params = _rand_params(ost.GPT_KEYS, 2, d, f, rng)
    lens = [1, 3, 5]
    xs = [rng.standard_normal((l, d)) for l in lens]
    dys = [rng.standard_normal((l, d)) for l in lens]
    outs, dxs, grads = ost.gpt_stage_fwd_bwd(xs, dys, params, h)
    eps = 1e-6
    # inputs
    for si in range(len(xs)):
        num = np.zeros_like(xs[si])
        for idx in np.ndindex(*xs[si].shape):
            old = xs[si][idx]
            xs[si][idx] = old + eps
            lp = _gpt_loss(xs, dys, params, h)
            xs[si][idx] = old - eps
            lm = _gpt_loss(xs, dys, params, h)
            xs[si][idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        assert np.abs(num - dxs[si]).max() <= 1e-6 * max(1.0, np.abs(num).max()), si
    # weights: every tensor, a spread of entries
    for li in range(2):
        for k in ost.GPT_KEYS:
            w = params[li][k]
            flat = list(np.ndindex(*w.shape))
            pick = [flat[i] for i in rng.choice(len(flat), size=min(10, len(flat)), replace=False)]
            for idx in pick:
                old = w[idx]
                w[idx] = old + eps
                lp = _gpt_loss(xs, dys, params, h)
                w[idx] = old - eps
                lm = _gpt_loss(xs, dys, params, h)
                w[idx] = old
                num = (lp - lm) / (2 * eps)
                assert abs(num - grads[li][k][idx]) <= 1e-6 * max(1.0, abs(num)), (li, k, idx)


def _t5_loss(ex, dx, ddy, ep, dp, h):
    outs = ost.t5_stage_fwd_bwd(ex, dx, ddy, ep, dp, h)[0]
    return sum(float((o * g).sum()) for o, g in zip(outs, ddy))


def test_t5_finite_differences():
    rng = np.random.default_rng(1)
    d, h, f = 8, 2, 10
    ep = _rand_params(ost.T5_ENC_KEYS, 1, d, f, rng)
    dp = _rand_params(ost.T5_DEC_KEYS, 2, d, f, rng)
    lin, ltg = [4, 2], [3, 1]
    ex = [rng.standard_normal((l, d)) for l in lin]
    dx = [rng.standard_normal((l, d)) for l in ltg]
    ddy = [rng.standard_normal((l, d)) for l in ltg]
    outs, d_enc, d_dec, eg, dg = ost.t5_stage_fwd_bwd(ex, dx, ddy, ep, dp, h)
    eps = 1e-6
    for arrs, grads_ in ((ex, d_enc), (dx, d_dec)):
        for si in range(2):
            for idx in np.ndindex(*arrs[si].shape):
                old = arrs[si][idx]
                arrs[si][idx] = old + eps
                lp = _t5_loss(ex, dx, ddy, ep, dp, h)
                arrs[si][idx] = old - eps
                lm = _t5_loss(ex, dx, ddy, ep, dp, h)
                arrs[si][idx] = old
                num = (lp - lm) / (2 * eps)
                assert abs(num - grads_[si][idx]) <= 1e-6 * max(1.0, abs(num))
    for plist, glist, keys in ((ep, eg, ost.T5_ENC_KEYS), (dp, dg, ost.T5_DEC_KEYS)):
        for li in range(len(plist)):
            for k in keys:
                w = plist[li][k]
                flat = list(np.ndindex(*w.shape))
                for idx in [flat[i] for i in rng.choice(len(flat), size=min(6, len(flat)), replace=False)]:
                    old = w[idx]
                    w[idx] = old + eps
                    lp = _t5_loss(ex, dx, ddy, ep, dp, h)
                    w[idx] = old - eps
                    lm = _t5_loss(ex, dx, ddy, ep, dp, h)
                    w[idx] = old
                    num = (lp - lm) / (2 * eps)
                    assert abs(num - glist[li][k][idx]) <= 1e-6 * max(1.0, abs(num)), (li, k, idx)


# ---------------------------------------------------------------- autograd library as a second opinion
def _t(a):
    return torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=True)


def _torch_attn(q, k, v, h, causal):
    lq, d = q.shape
    lk = k.shape[0]
    hd = d // h
    qh = q.view(lq, h, hd).transpose(0, 1)
    kh = k.view(lk, h, hd).transpose(0, 1)
    vh = v.view(lk, h, hd).transpose(0, 1)
    o = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh, is_causal=causal)
    return o.transpose(0, 1).reshape(lq, d)


def _torch_gpt_layer(x, p, h):
    F = torch.nn.functional
    d = x.shape[1]
    u1 = F.layer_norm(x, (d,), p["ln1_g"], p["ln1_b"], eps=1e-5)
    qkv = F.linear(u1, p["w_qkv"].t(), p["b_qkv"])
    o = _torch_attn(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], h, True)
    x1 = x + F.linear(o, p["w_o"].t(), p["b_o"])
    u2 = F.layer_norm(x1, (d,), p["ln2_g"], p["ln2_b"], eps=1e-5)
    a = F.gelu(F.linear(u2, p["w_1"].t(), p["b_1"]), approximate="tanh")
    return x1 + F.linear(a, p["w_2"].t(), p["b_2"])


def test_gpt_against_autograd_library():
    rng = np.random.default_rng(2)
    d, h, f = 32, 4, 48
    params = _rand_params(ost.GPT_KEYS, 2, d, f, rng, std=0.2)
    lens = [1, 7, 20, 13]
    xs = [rng.standard_normal((l, d)) for l in lens]
    dys = [rng.standard_normal((l, d)) for l in lens]
    outs, dxs, grads = ost.gpt_stage_fwd_bwd(xs, dys, params, h)
    tp = [{k: _t(v) for k, v in layer.items()} for layer in params]
    txs = [_t(x) for x in xs]
    loss = 0
    touts = []
    for x, dy in zip(txs, dys):
        y = x
        for p in tp:
            y = _torch_gpt_layer(y, p, h)
        touts.append(y)
        loss = loss + (y * torch.tensor(dy)).sum()
    loss.backward()
    for o, to in zip(outs, touts):
        np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-10, atol=1e-10)
    for dx, tx in zip(dxs, txs):
        np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-10)
    for li in range(2):
        for k in ost.GPT_KEYS:
            np.testing.assert_allclose(grads[li][k], tp[li][k].grad.numpy(), rtol=1e-9, atol=1e-10, err_msg=k)


def _torch_rms(x, g):
    return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-6) * g


def _torch_t5_mlp(x, p):
    u = _torch_rms(x, p["ln2_g"])
    a = torch.nn.functional.gelu(u @ p["w_g"], approximate="tanh") * (u @ p["w_u"])
    return x + a @ p["w_2"]


def test_t5_against_autograd_library():
    rng = np.random.default_rng(4)
    d, h, f = 16, 2, 24
    ep = _rand_params(ost.T5_ENC_KEYS, 2, d, f, rng, std=0.2)
    dp = _rand_params(ost.T5_DEC_KEYS, 2, d, f, rng, std=0.2)
    lin, ltg = [9, 2, 5], [4, 6, 1]
    ex = [rng.standard_normal((l, d)) for l in lin]
    dx = [rng.standard_normal((l, d)) for l in ltg]
    ddy = [rng.standard_normal((l, d)) for l in ltg]
    outs, d_enc, d_dec, eg, dg = ost.t5_stage_fwd_bwd(ex, dx, ddy, ep, dp, h)
    tep = [{k: _t(v) for k, v in layer.items()} for layer in ep]
    tdp = [{k: _t(v) for k, v in layer.items()} for layer in dp]
    tex, tdx = [_t(a) for a in ex], [_t(a) for a in dx]
    loss = 0
    touts = []
    for e, y, g in zip(tex, tdx, ddy):
        for p in tep:
            u = _torch_rms(e, p["ln1_g"])
            qkv = u @ p["w_qkv"]
            e = e + _torch_attn(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], h, False) @ p["w_o"]
            e = _torch_t5_mlp(e, p)
        for p in tdp:
            u = _torch_rms(y, p["ln1_g"])
            qkv = u @ p["w_qkv"]
            y = y + _torch_attn(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], h, True) @ p["w_o"]
            u = _torch_rms(y, p["lnc_g"])
            kv = e @ p["w_ckv"]
            y = y + _torch_attn(u @ p["w_cq"], kv[:, :d], kv[:, d:], h, False) @ p["w_co"]
            y = _torch_t5_mlp(y, p)
        touts.append(y)
        loss = loss + (y * torch.tensor(g)).sum()
    loss.backward()
    for o, to in zip(outs, touts):
        np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-10, atol=1e-10)
    for a, t in zip(d_enc + d_dec, tex + tdx):
        np.testing.assert_allclose(a, t.grad.numpy(), rtol=1e-9, atol=1e-10)
    for plist, glist in ((tep, eg), (tdp, dg)):
        for li in range(2):
            for k in plist[li]:
                np.testing.assert_allclose(glist[li][k], plist[li][k].grad.numpy(), rtol=1e-9, atol=1e-10, err_msg=k)


# ---------------------------------------------------------------- closed forms
def test_single_token_attention_returns_value_row():
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((1, 8)) for _ in range(3))
    for causal in (True, False):
        o, _ = ost.attention_fwd(q, k, v, 2, causal)
        np.testing.assert_allclose(o, v, rtol=0, atol=1e-15)


def test_first_causal_token_sees_only_itself_and_uniform_scores_average():
    rng = np.random.default_rng(6)
    l, d = 6, 8
    q = rng.standard_normal((l, d))
    k = rng.standard_normal((l, d))
    v = rng.standard_normal((l, d))
    o, _ = ost.attention_fwd(q, k, v, 2, True)
    np.testing.assert_allclose(o[0], v[0], atol=1e-15)
    # zero queries: uniform probabilities, so causal row i is the mean of v[0..i], bidirectional the full mean
    oc, _ = ost.attention_fwd(np.zeros_like(q), k, v, 2, True)
    ob, _ = ost.attention_fwd(np.zeros_like(q), k, v, 2, False)
    for i in range(l):
        np.testing.assert_allclose(oc[i], v[:i + 1].mean(axis=0), atol=1e-14)
        np.testing.assert_allclose(ob[i], v.mean(axis=0), atol=1e-14)


def test_zero_projections_make_the_block_the_identity():
    rng = np.random.default_rng(7)
    d, h, f = 8, 2, 12
    params = _rand_params(ost.GPT_KEYS, 1, d, f, rng)
    for k in ("w_o", "b_o", "w_2", "b_2"):
        params[0][k][...] = 0.0
    x = rng.standard_normal((5, d))
    out = ost.gpt_stage_fwd([x], params, h)[0]
    np.testing.assert_allclose(out, x, atol=0)


def test_norms_on_special_rows():
    g = np.array([1.5, -2.0, 0.5, 3.0])
    b = np.array([0.1, 0.2, 0.3, 0.4])
    y, _ = ost.layernorm_fwd(np.full((2, 4), 7.0), g, b)
    np.testing.assert_allclose(y, np.tile(b, (2, 1)), atol=1e-12)      # constant row -> bias
    x = np.array([[1.0, -1.0, 1.0, -1.0]])
    y, _ = ost.layernorm_fwd(x, g, b)                                   # mean 0, variance 1
    np.testing.assert_allclose(y, x / math.sqrt(1 + 1e-5) * g + b, atol=1e-15)
    y, _ = ost.rmsnorm_fwd(np.array([[3.0, 4.0, 0.0, 0.0]]), g)         # mean square 25/4
    np.testing.assert_allclose(y, np.array([[3.0, 4.0, 0, 0]]) / math.sqrt(6.25 + 1e-6) * g, atol=1e-15)


def test_gelu_values():
    np.testing.assert_allclose(ost.gelu(np.array([0.0])), [0.0])
    np.testing.assert_allclose(ost.gelu(np.array([10.0, -10.0])), [10.0, 0.0], atol=1e-12)
    z = 1.0
    ref = 0.5 * z * (1 + math.tanh(math.sqrt(2 / math.pi) * (z + 0.044715)))
    np.testing.assert_allclose(ost.gelu(np.array([z])), [ref], rtol=1e-15)
    np.testing.assert_allclose(ost.gelu_grad(np.array([0.0])), [0.5])


def test_sequences_are_independent_and_weight_grads_add():
    rng = np.random.default_rng(8)
    d, h, f = 16, 4, 24
    params = _rand_params(ost.GPT_KEYS, 2, d, f, rng)
    lens = [3, 9, 4]
    xs = [rng.standard_normal((l, d)) for l in lens]
    dys = [rng.standard_normal((l, d)) for l in lens]
    outs, dxs, grads = ost.gpt_stage_fwd_bwd(xs, dys, params, h)
    acc = None
    for i in range(3):
        o1, dx1, g1 = ost.gpt_stage_fwd_bwd([xs[i]], [dys[i]], params, h)
        np.testing.assert_array_equal(o1[0], outs[i])
        np.testing.assert_array_equal(dx1[0], dxs[i])
        if acc is None:
            acc = g1
        else:
            for li in range(2):
                for k in g1[li]:
                    acc[li][k] = acc[li][k] + g1[li][k]
    for li in range(2):
        for k in acc[li]:
            np.testing.assert_allclose(acc[li][k], grads[li][k], rtol=1e-12, atol=1e-13)
