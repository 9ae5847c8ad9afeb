"""The flop accounting behind the benchmark's utilisation figures, against counts written out the long way (host only)."""
import numpy as np
import pytest

import bench


def _count_gpt(d, F, L, lens):
    """Multiply-adds x 2 of one decoder-only stage, forward, operation by operation, then x 3 for forward + backward
    (every product has two gradient products of its own size)."""
    linear = attn = 0
    for _ in range(L):
        for l in lens:
            for _tok in range(int(l)):
                linear += 2 * d * 3 * d        # QKV projection of one token
                linear += 2 * d * d            # attention output projection
                linear += 2 * d * F            # first MLP projection
                linear += 2 * F * d            # second MLP projection
            for i in range(int(l)):            # query i sees keys 0..i: a score and a weighted value row per pair, all heads
                attn += 2 * d * (i + 1)        # q . k over d = heads x head_dim
                attn += 2 * d * (i + 1)        # p x v
    return 3 * linear, 3 * attn


def _count_t5(d, F, L, Ld, lens, tgts):
    linear = attn = 0
    for _ in range(L):                          # encoder layer: QKV, output, two gate/up projections, down projection
        for l in lens:
            linear += int(l) * (2 * d * 3 * d + 2 * d * d + 2 * (2 * d * F) + 2 * F * d)
            attn += 2 * (2 * d * int(l) * int(l))            # bidirectional: every pair, scores and values
    for _ in range(Ld):                         # decoder layer: self-attention, cross-attention (Q, output on target
        for l, t in zip(lens, tgts):            # tokens; K, V on encoder tokens), gated MLP
            l, t = int(l), int(t)
            linear += t * (2 * d * 3 * d + 2 * d * d)
            linear += t * (2 * d * d + 2 * d * d) + l * (2 * d * 2 * d)
            linear += t * (2 * (2 * d * F) + 2 * F * d)
            attn += 2 * sum(2 * d * (i + 1) for i in range(t))
            attn += 2 * (2 * d * t * l)
    return 3 * linear, 3 * attn


@pytest.mark.parametrize("seed", range(4))
def test_algorithmic_flops_count_every_product(seed):
    rng = np.random.default_rng(seed)
    d, F, L = 8 * int(rng.integers(1, 5)), 8 * int(rng.integers(1, 9)), int(rng.integers(1, 4))
    lens = rng.integers(1, 40, int(rng.integers(1, 9)))
    cfg = {"kind": "gpt", "d_model": d, "d_ff": F, "n_layers": L}
    assert bench.algorithmic_flops(cfg, lens) == _count_gpt(d, F, L, lens)
    tgts = rng.integers(1, 30, len(lens))
    cfg = {"kind": "t5", "d_model": d, "d_ff": F, "n_layers": L, "n_dec_layers": L + 1}
    assert bench.algorithmic_flops(cfg, lens, tgts) == _count_t5(d, F, L, L + 1, lens, tgts)


def _needed_blocks(ql, kl, causal):
    """32 x 32 score blocks that hold at least one (query, key) pair the method needs."""
    n = 0
    for q0 in range(0, ql, 32):
        for k0 in range(0, kl, 32):
            if not causal or k0 <= min(ql - 1, q0 + 31):
                n += 1
    return n


@pytest.mark.parametrize("causal", [False, True])
def test_executed_attention_blocks_cover_the_needed_ones_and_no_more_than_the_padded_rectangle(causal):
    rng = np.random.default_rng(7 + causal)
    cases = [(1, 1), (32, 32), (33, 64), (128, 128), (129, 129), (64, 300), (300, 64), (511, 511), (640, 640)]
    cases += [(int(a), int(b)) for a, b in rng.integers(1, 700, (40, 2))]
    for ql, kl in cases:
        if causal:
            kl = ql                                             # causal attention here is self-attention
        fwd, dq, dkv = bench.attention_tiles(ql, kl, causal)
        need = _needed_blocks(ql, kl, causal)
        full = ((ql + 127) // 128 * 4) * ((kl + 63) // 64 * 2)  # query blocks of 128, key tiles of 64
        assert need <= dq <= fwd <= full, (ql, kl, causal, need, dq, fwd, full)
        full_kv = ((kl + 127) // 128 * 4) * ((ql + 63) // 64 * 2)
        assert need <= dkv <= full_kv, (ql, kl, causal, need, dkv, full_kv)
    assert bench.attention_tiles(0, 5, causal) == (0, 0, 0) and bench.attention_tiles(5, 0, causal) == (0, 0, 0)


def test_attention_blocks_of_whole_tiles_without_mask_are_the_rectangle():
    for ql, kl in [(128, 64), (256, 512), (384, 128)]:
        n = (ql // 32) * (kl // 32)
        assert bench.attention_tiles(ql, kl, False) == (n, n, n)


class _Layout:
    def __init__(self, rows, rows_tgt=0):
        self.total_rows, self.total_rows_tgt = rows, rows_tgt


def test_executed_flops_are_never_below_the_algorithmic_ones():
    rng = np.random.default_rng(3)
    d, F, L = 64, 256, 2
    lens = np.sort(rng.integers(1, 600, 12))
    cfg = {"kind": "gpt", "d_model": d, "d_ff": F, "n_layers": L}
    lin_a, att_a = bench.algorithmic_flops(cfg, lens)
    lin_e, att_e = bench.executed_flops(cfg, _Layout(int(lens.sum())), lens, None)
    assert lin_e == lin_a and att_e >= att_a                   # no padding rows: the projections match exactly
    lin_p, _ = bench.executed_flops(cfg, _Layout(int(lens.sum()) + 100), lens, None)
    assert lin_p == lin_a + 3 * 2 * (4 * d * d + 2 * d * F) * 100 * L
    tgts = rng.integers(1, 200, len(lens))
    cfg = {"kind": "t5", "d_model": d, "d_ff": F, "n_layers": L, "n_dec_layers": 2}
    lin_a, att_a = bench.algorithmic_flops(cfg, lens, tgts)
    lin_e, att_e = bench.executed_flops(cfg, _Layout(int(lens.sum()), int(tgts.sum())), lens, tgts)
    assert lin_e == lin_a and att_e >= att_a
