"""Seeded synthetic inputs: sequence lengths, weights, activations, upstream gradients.

This module holds none of the method's arithmetic (no cost model, no partitioning, no layer
math): it only draws random numbers in a fixed call order, so that the CPU oracle used by the
tests and the HIP path can be fed the same values.  The length distributions stand in for the
paper's FLANv2 workload (section "Evaluation", dataset paragraph): heavy right tail, global
batch of about 65536 tokens, maximum lengths 512..8192.
"""
import numpy as np

GPT_KEYS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")
T5_ENC_KEYS = ("ln1_g", "w_qkv", "w_o", "ln2_g", "w_g", "w_u", "w_2")
T5_DEC_KEYS = ("ln1_g", "w_qkv", "w_o", "lnc_g", "w_cq", "w_ckv", "w_co", "ln2_g", "w_g", "w_u", "w_2")

CONFIGS = {
    # name: model + workload description (shapes follow the five configurations of the build's baseline file)
    "gpt_small_fp32": dict(kind="gpt", dtype="f32", n_layers=2, d_model=256, n_heads=4, d_ff=1024,
                           lengths=dict(rule="count", count=64, mu=4.5, sigma=0.8, lo=8, hi=512),
                           num_stages=4, cap=4096),
    "gpt_2048_bf16": dict(kind="gpt", dtype="bf16", n_layers=4, d_model=2048, n_heads=16, d_ff=8192,
                          lengths=dict(rule="tokens", tokens=65536, mu=5.5, sigma=1.0, lo=16, hi=2048),
                          num_stages=4, cap=16384),
    "t5_1024_bf16": dict(kind="t5", dtype="bf16", n_layers=2, n_dec_layers=2, d_model=1024, n_heads=16, d_ff=2816,
                         lengths=dict(rule="tokens", tokens=65536, mu=5.3, sigma=1.0, lo=8, hi=2048,
                                      tgt_mu=3.5, tgt_sigma=1.0, tgt_lo=1, tgt_hi=512),
                         num_stages=4, cap=16384),
    "gpt_4096_longtail_bf16": dict(kind="gpt", dtype="bf16", n_layers=2, d_model=4096, n_heads=32, d_ff=16384,
                                   lengths=dict(rule="tokens_bimodal", tokens=131072, p_short=0.7,
                                                mu=4.5, sigma=0.7, mu2=7.5, sigma2=0.5, lo=16, hi=8192),
                                   num_stages=8, cap=32768),
}


def _clip_round(v, lo, hi):
    return int(min(max(int(np.rint(v)), lo), hi))


def draw_lengths(spec, seed=0):
    """Return (lengths, lengths_tgt or None) as int32 arrays; one scalar draw per call, in a fixed order."""
    rng = np.random.default_rng([seed, 1])
    lens, tgts = [], []
    has_tgt = "tgt_mu" in spec

    def one():
        if spec["rule"] == "tokens_bimodal":
            u = rng.random()
            if u < spec["p_short"]:
                v = rng.lognormal(spec["mu"], spec["sigma"])
            else:
                v = rng.lognormal(spec["mu2"], spec["sigma2"])
        else:
            v = rng.lognormal(spec["mu"], spec["sigma"])
        lens.append(_clip_round(v, spec["lo"], spec["hi"]))
        if has_tgt:
            t = rng.lognormal(spec["tgt_mu"], spec["tgt_sigma"])
            tgts.append(_clip_round(t, spec["tgt_lo"], spec["tgt_hi"]))

    if spec["rule"] == "count":
        for _ in range(spec["count"]):
            one()
    else:
        total = 0
        while total < spec["tokens"]:
            one()
            total += lens[-1]
    return np.asarray(lens, dtype=np.int32), (np.asarray(tgts, dtype=np.int32) if has_tgt else None)


def to_bf16_grid(a):
    """Round float32 values to the nearest bfloat16 (ties to even) and return them as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def _shape_of(key, d, f):
    return {
        "ln1_g": (d,), "ln1_b": (d,), "ln2_g": (d,), "ln2_b": (d,), "lnc_g": (d,),
        "w_qkv": (d, 3 * d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
        "w_1": (d, f), "b_1": (f,), "w_2": (f, d), "b_2": (d,),
        "w_g": (d, f), "w_u": (d, f),
        "w_cq": (d, d), "w_ckv": (d, 2 * d), "w_co": (d, d),
    }[key]


def draw_params(keys, n_layers, d_model, d_ff, seed=0, tag=2, bf16=False, std=0.02):
    """Per layer a dict key -> float32 array.  Matrices, biases ~ N(0, std); gains ~ 1 + N(0, std)."""
    layers = []
    for li in range(n_layers):
        layer = {}
        for ki, key in enumerate(keys):
            rng = np.random.default_rng([seed, tag, li, ki])
            v = rng.standard_normal(_shape_of(key, d_model, d_ff), dtype=np.float32) * np.float32(std)
            if key.endswith("_g") and key.startswith("ln"):
                v = v + np.float32(1.0)
            layer[key] = to_bf16_grid(v) if bf16 else v
        layers.append(layer)
    return layers


def draw_rows(lengths, d_model, seed=0, tag=3, bf16=False):
    """One [l_i, d] float32 array of N(0,1) values per sequence (original sample order)."""
    out = []
    for i, l in enumerate(lengths):
        rng = np.random.default_rng([seed, tag, i])
        v = rng.standard_normal((int(l), d_model), dtype=np.float32)
        out.append(to_bf16_grid(v) if bf16 else v)
    return out


def draw_embedded_tokens(lengths, d_model, vocab=32000, seed=0, tag=4, bf16=False):
    """Token ids uniform in [0, vocab) looked up in a random N(0,1) table (the stage input of the small config)."""
    rng = np.random.default_rng([seed, tag, 0])
    table = rng.standard_normal((vocab, d_model), dtype=np.float32)
    if bf16:
        table = to_bf16_grid(table)
    out = []
    for i, l in enumerate(lengths):
        r = np.random.default_rng([seed, tag, 1, i])
        ids = r.integers(0, vocab, size=int(l))
        out.append(table[ids].copy())
    return out
