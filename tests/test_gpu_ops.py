"""GPU parity of the building-block kernels, each called through the C ABI and compared with its plain
definition (numpy float64 on the same rounded inputs, or the oracle's per-sequence attention / norm
functions).  Every comparison bounds the normwise relative error by the stated tolerance AND every
single element's deviation by tolerance x (8 x rms(reference) + |reference element|) (helpers.both_err).  Sizes span several
tiles and a ragged tail."""
import numpy as np
import pytest
import torch

from oracle import stage as ost
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl
from helpers import DEV, both_err, to_dev, to_np

pytestmark = pytest.mark.gpu

BF, F32 = torch.bfloat16, torch.float32
TOL = {BF: 2e-2, F32: 1e-4}


def _rnd(rng, shape, dt, scale=1.0):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    if dt == BF:
        a = wl.to_bf16_grid(a)
    return a


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, True), (BF, False)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False)])
def test_gemm_plain(dt, force, ta, tb):
    rng = np.random.default_rng(1)
    if ta:
        M, N, K = 512, 768, 1000 + 37          # weight-gradient shape: ragged contraction over tokens
    else:
        M, N, K = 1000 + 37, 512, 320           # ragged M, several K steps
    A = _rnd(rng, (K, M) if ta else (M, K), dt)
    B = _rnd(rng, (N, K) if tb else (K, N), dt)
    bias = _rnd(rng, (N,), dt)
    ref = (A.T if ta else A).astype(np.float64) @ (B.T if tb else B).astype(np.float64) + bias
    dA, dB, db = to_dev(A, dt), to_dev(B, dt), to_dev(bias, dt)
    Cd = torch.zeros((M, N), dtype=dt, device=DEV)
    ds.ds_gemm(dA, dB, Cd, M, N, K, trans_a=ta, trans_b=tb, bias=db, force_generic=force)
    torch.cuda.synchronize()
    # bf16 output rounding: 2^-9 relative per element
    assert both_err(to_np(Cd), ref) <= (4e-3 if dt == BF else 1e-5)


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, False)])
def test_gemm_epilogues(dt, force):
    rng = np.random.default_rng(2)
    M, N, K = 700, 256, 128
    A, B = _rnd(rng, (M, K), dt), _rnd(rng, (K, N), dt, 0.1)
    bias, R = _rnd(rng, (N,), dt), _rnd(rng, (M, N), dt)
    R2 = _rnd(rng, (M, N), dt)
    valid = np.where(rng.random(M) < 0.8, 1, -1).astype(np.int32)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    dA, dB, db, dR, dR2 = (to_dev(x, dt) for x in (A, B, bias, R, R2))
    dvalid = torch.from_numpy(valid).to(DEV)
    tol = 6e-3 if dt == BF else 1e-5

    def run(epi, **kw):
        c = torch.zeros((M, N), dtype=dt, device=DEV)
        c2 = torch.zeros((M, N), dtype=dt, device=DEV)
        ds.ds_gemm(dA, dB, c, M, N, K, epilogue=epi, C2=c2, force_generic=force, **kw)
        torch.cuda.synchronize()
        return to_np(c), to_np(c2)

    z, a = run(ds.DS_EPI_GELU, bias=db)
    assert both_err(z, acc + bias) <= tol and both_err(a, ost.gelu(acc + bias)) <= tol
    c, _ = run(ds.DS_EPI_RESID, bias=db, R=dR, row_valid=dvalid)
    ref = (acc + bias + R) * (valid[:, None] >= 0)
    assert both_err(c, ref) <= tol and np.all(c[valid < 0] == 0)
    c, _ = run(ds.DS_EPI_DGELU, R=dR)
    assert both_err(c, acc * ost.gelu_grad(R.astype(np.float64))) <= tol
    gd, a = run(ds.DS_EPI_GELU_D, bias=db)                # derivative kept instead of the pre-activation
    assert both_err(gd, ost.gelu_grad(acc + bias)) <= tol and both_err(a, ost.gelu(acc + bias)) <= tol
    c, _ = run(ds.DS_EPI_MULR, R=dR)
    assert both_err(c, acc * R) <= tol
    zu, h = run(ds.DS_EPI_GATE, R=dR)
    assert both_err(zu, acc) <= tol and both_err(h, ost.gelu(R.astype(np.float64)) * acc) <= tol
    g1, g2 = run(ds.DS_EPI_DGATE, R=dR, R2=dR2)
    assert both_err(g1, acc * R2 * ost.gelu_grad(R.astype(np.float64))) <= tol
    assert both_err(g2, acc * ost.gelu(R.astype(np.float64))) <= tol


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, False)])
@pytest.mark.parametrize("M,N,K", [(256, 512, 3000 + 11), (768, 512, 1000 + 37), (512, 256, 31), (256, 256, 64)])
def test_gemm_weight_gradient_accumulates_in_fp32(dt, force, M, N, K):
    rng = np.random.default_rng(3)
    X, dY = _rnd(rng, (K, M), dt), _rnd(rng, (K, N), dt)
    ref = X.astype(np.float64).T @ dY.astype(np.float64)
    dX, ddY = to_dev(X, dt), to_dev(dY, dt)
    Cd = torch.full((M, N), 3.0, dtype=F32, device=DEV)
    ds.ds_gemm(dX, ddY, Cd, M, N, K, trans_a=True, epilogue=ds.DS_EPI_ACC32, accumulate=False, force_generic=force)
    ds.ds_gemm(dX, ddY, Cd, M, N, K, trans_a=True, epilogue=ds.DS_EPI_ACC32, accumulate=True, force_generic=force)
    torch.cuda.synchronize()
    assert both_err(to_np(Cd), 2 * ref) <= 1e-5


def _varlen_case(rng, lens, h, hd, dt, cross_lens=None):
    d = h * hd
    T = int(sum(lens)) + 5                       # 5 trailing rows never touched
    gap = 3
    rows, r = [], 0
    for l in lens:
        rows.append(r)
        r += l + gap                              # gaps play the role of padding rows
    T = r + 2
    qkv = _rnd(rng, (T, 3 * d), dt)
    d_o = _rnd(rng, (T, d), dt)
    return d, T, np.asarray(rows, np.int32), qkv, d_o


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, True), (BF, False)])
@pytest.mark.parametrize("hd,causal", [(64, True), (128, True), (64, False), (128, False)])
def test_attention_self(dt, force, hd, causal):
    rng = np.random.default_rng(4)
    h = 2
    # lengths on both sides of every tile boundary (64-row steps, 128-row blocks), a few long ones for the middle steps
    lens = [1, 7, 63, 64, 65, 127, 128, 129, 130, 191, 192, 193, 200, 256, 257, 333, 700]
    d, T, rows, qkv, d_o = _varlen_case(rng, lens, h, hd, dt)
    dq = to_dev(qkv, dt)
    o = torch.zeros((T, d), dtype=dt, device=DEV)
    lse = torch.zeros((h, T), dtype=F32, device=DEV)
    delta = torch.zeros((h, T), dtype=F32, device=DEV)
    dqkv = torch.zeros((T, 3 * d), dtype=dt, device=DEV)
    ddo = to_dev(d_o, dt)
    # the sequence table is handed over in an arbitrary order: nothing may depend on ascending rows
    order = rng.permutation(len(lens))
    t_rows = torch.from_numpy(np.ascontiguousarray(rows[order])).to(DEV)
    t_lens = torch.tensor([lens[i] for i in order], dtype=torch.int32, device=DEV)
    scratch = torch.zeros(ds.ds_attention_scratch_bytes(h, hd, T, T, len(lens)), dtype=torch.uint8, device=DEV)
    es = dq.element_size()
    base = dq.data_ptr()
    ds.ds_attention_fwd(base, base + d * es, base + 2 * d * es, o, lse, t_rows, t_lens, t_rows, t_lens, h, hd, causal,
                        max(lens), max(lens), 3 * d, 3 * d, 3 * d, d, T, scratch=scratch, force_generic=force)
    gb = dqkv.data_ptr()
    ds.ds_attention_bwd(base, base + d * es, base + 2 * d * es, o, ddo, lse, delta, gb, gb + d * es, gb + 2 * d * es,
                        t_rows, t_lens, t_rows, t_lens, h, hd, causal, max(lens), max(lens), 3 * d, 3 * d, 3 * d, d, T,
                        scratch=scratch, force_generic=force)
    torch.cuda.synchronize()
    o_np, g_np, lse_np = to_np(o), to_np(dqkv), to_np(lse)
    tol = TOL[dt]
    touched = np.zeros(T, dtype=bool)
    for r0, l in zip(rows, lens):
        x = qkv[r0:r0 + l].astype(np.float64)
        q, k, v = x[:, :d], x[:, d:2 * d], x[:, 2 * d:]
        ref_o, cache = ost.attention_fwd(q, k, v, h, causal)
        # the backward kernels consume the ROUNDED forward output, as the oracle's gradient of the exact one
        rq, rk, rv = ost.attention_bwd(d_o[r0:r0 + l].astype(np.float64), cache)
        assert both_err(o_np[r0:r0 + l], ref_o) <= tol, (l, "o")
        assert both_err(g_np[r0:r0 + l, :d], rq) <= tol, (l, "dq")
        assert both_err(g_np[r0:r0 + l, d:2 * d], rk) <= tol, (l, "dk")
        assert both_err(g_np[r0:r0 + l, 2 * d:], rv) <= tol, (l, "dv")
        # log-sum-exp of the scaled scores, head 0, last row
        s = (q[-1, :hd] @ k[:, :hd].T) / np.sqrt(hd)      # the last query sees every key in both mask kinds
        assert abs(lse_np[0, r0 + l - 1] - np.log(np.exp(s - s.max()).sum()) - s.max()) <= 2e-2
        touched[r0:r0 + l] = True
    assert np.all(o_np[~touched] == 0) and np.all(g_np[~touched] == 0)      # padding rows are never written


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, False)])
def test_attention_cross(dt, force):
    rng = np.random.default_rng(5)
    h, hd = 2, 64
    d = h * hd
    ql, kl = [3, 40, 129, 200, 64], [70, 5, 260, 700, 1000]      # the last two: many key steps / many query steps per block
    qr = np.array([0, 5, 50, 190, 400], np.int32)
    kr = np.array([2, 80, 90, 360, 1070], np.int32)
    Tq, Tk = 470, 2080
    q = _rnd(rng, (Tq, d), dt)
    kv = _rnd(rng, (Tk, 2 * d), dt)
    d_o = _rnd(rng, (Tq, d), dt)
    tq, tkv, tdo = to_dev(q, dt), to_dev(kv, dt), to_dev(d_o, dt)
    o = torch.zeros((Tq, d), dtype=dt, device=DEV)
    lse = torch.zeros((h, Tq), dtype=F32, device=DEV)
    delta = torch.zeros((h, Tq), dtype=F32, device=DEV)
    dq = torch.zeros((Tq, d), dtype=dt, device=DEV)
    dkv = torch.zeros((Tk, 2 * d), dtype=dt, device=DEV)
    es = tq.element_size()
    i32 = lambda a: torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    t_qr, t_ql, t_kr, t_kl = i32(qr), i32(ql), i32(kr), i32(kl)
    kb = tkv.data_ptr()
    scratch = torch.zeros(ds.ds_attention_scratch_bytes(h, hd, Tq, Tk, len(ql)), dtype=torch.uint8, device=DEV)
    ds.ds_attention_fwd(tq, kb, kb + d * es, o, lse, t_qr, t_ql, t_kr, t_kl, h, hd, False, max(ql), max(kl),
                        d, 2 * d, 2 * d, d, Tq, k_total_rows=Tk, scratch=scratch, force_generic=force)
    gb = dkv.data_ptr()
    ds.ds_attention_bwd(tq, kb, kb + d * es, o, tdo, lse, delta, dq, gb, gb + d * es, t_qr, t_ql, t_kr, t_kl, h, hd, False,
                        max(ql), max(kl), d, 2 * d, 2 * d, d, Tq, k_total_rows=Tk, scratch=scratch, force_generic=force)
    torch.cuda.synchronize()
    tol = TOL[dt]
    for i in range(len(ql)):
        qq = q[qr[i]:qr[i] + ql[i]].astype(np.float64)
        kk = kv[kr[i]:kr[i] + kl[i], :d].astype(np.float64)
        vv = kv[kr[i]:kr[i] + kl[i], d:].astype(np.float64)
        ref_o, cache = ost.attention_fwd(qq, kk, vv, h, False)
        rq, rk, rv = ost.attention_bwd(d_o[qr[i]:qr[i] + ql[i]].astype(np.float64), cache)
        assert both_err(to_np(o)[qr[i]:qr[i] + ql[i]], ref_o) <= tol
        assert both_err(to_np(dq)[qr[i]:qr[i] + ql[i]], rq) <= tol
        assert both_err(to_np(dkv)[kr[i]:kr[i] + kl[i], :d], rk) <= tol
        assert both_err(to_np(dkv)[kr[i]:kr[i] + kl[i], d:], rv) <= tol


@pytest.mark.parametrize("dt,force", [(F32, True), (BF, True), (BF, False)])
def test_attention_empty_sequences(dt, force):
    """q_len = 0: the sequence is skipped.  k_len = 0: its outputs and query gradients are zero, and nothing is
    fetched for it (its key rows are given as row 0 of the tensor, where a fetch of the row before would fall
    outside the allocation)."""
    rng = np.random.default_rng(15)
    h, hd = 2, 64
    d = h * hd
    ql, kl = [0, 37, 130], [50, 0, 140]
    qr = np.array([0, 4, 60], np.int32)
    kr = np.array([10, 0, 70], np.int32)
    Tq, Tk = 200, 220
    q = _rnd(rng, (Tq, d), dt)
    kv = _rnd(rng, (Tk, 2 * d), dt)
    d_o = _rnd(rng, (Tq, d), dt)
    tq, tkv, tdo = to_dev(q, dt), to_dev(kv, dt), to_dev(d_o, dt)
    o = torch.full((Tq, d), 7.0, dtype=dt, device=DEV)
    lse = torch.zeros((h, Tq), dtype=F32, device=DEV)
    delta = torch.zeros((h, Tq), dtype=F32, device=DEV)
    dq = torch.full((Tq, d), 7.0, dtype=dt, device=DEV)
    dkv = torch.zeros((Tk, 2 * d), dtype=dt, device=DEV)
    es = tq.element_size()
    i32 = lambda a: torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    t_qr, t_ql, t_kr, t_kl = i32(qr), i32(ql), i32(kr), i32(kl)
    kb = tkv.data_ptr()
    scratch = torch.zeros(ds.ds_attention_scratch_bytes(h, hd, Tq, Tk, 3), dtype=torch.uint8, device=DEV)
    ds.ds_attention_fwd(tq, kb, kb + d * es, o, lse, t_qr, t_ql, t_kr, t_kl, h, hd, False, max(ql), max(kl),
                        d, 2 * d, 2 * d, d, Tq, k_total_rows=Tk, scratch=scratch, force_generic=force)
    gb = dkv.data_ptr()
    ds.ds_attention_bwd(tq, kb, kb + d * es, o, tdo, lse, delta, dq, gb, gb + d * es, t_qr, t_ql, t_kr, t_kl, h, hd, False,
                        max(ql), max(kl), d, 2 * d, 2 * d, d, Tq, k_total_rows=Tk, scratch=scratch, force_generic=force)
    torch.cuda.synchronize()
    o_np, dq_np, dkv_np = to_np(o), to_np(dq), to_np(dkv)
    tol = TOL[dt]
    # the sequence without keys: zeros; rows of no sequence (and of the one without queries): untouched
    assert np.all(o_np[4:4 + 37] == 0) and np.all(dq_np[4:4 + 37] == 0)
    untouched = np.ones(Tq, dtype=bool)
    untouched[4:4 + 37] = False
    untouched[60:60 + 130] = False
    assert np.all(o_np[untouched] == 7.0) and np.all(dq_np[untouched] == 7.0)
    assert np.all(dkv_np[:70] == 0) and np.all(dkv_np[70 + 140:] == 0)       # keys of the query-less sequence get nothing
    # the ordinary sequence beside them is unaffected
    qq = q[60:190].astype(np.float64)
    kk = kv[70:210, :d].astype(np.float64)
    vv = kv[70:210, d:].astype(np.float64)
    ref_o, cache = ost.attention_fwd(qq, kk, vv, h, False)
    rq, rk, rv = ost.attention_bwd(d_o[60:190].astype(np.float64), cache)
    assert both_err(o_np[60:190], ref_o) <= tol
    assert both_err(dq_np[60:190], rq) <= tol
    assert both_err(dkv_np[70:210, :d], rk) <= tol
    assert both_err(dkv_np[70:210, d:], rv) <= tol


@pytest.mark.parametrize("dt", [F32, BF])
@pytest.mark.parametrize("rms", [False, True])
@pytest.mark.parametrize("d", [256, 1024, 1536, 2048, 3072, 4096])
def test_norm_forward_backward(dt, rms, d):
    _norm_case(dt, rms, d, 1000 + 3)


@pytest.mark.parametrize("dt,rms", [(BF, False), (F32, True)])
def test_norm_wide_rows_more_rows_than_work_groups(dt, rms):
    """d = 4096 runs a pair of wavefronts per row; with more rows than work-groups each pair walks several rows."""
    _norm_case(dt, rms, 4096, 4500)


def _norm_case(dt, rms, d, rows):
    rng = np.random.default_rng(6)
    x = _rnd(rng, (rows, d), dt, 2.0) + (0 if rms else 0.5)
    if dt == BF:
        x = wl.to_bf16_grid(x)
    g = _rnd(rng, (d,), dt, 0.1) + 1.0
    if dt == BF:
        g = wl.to_bf16_grid(g)
    b = _rnd(rng, (d,), dt, 0.1)
    dy = _rnd(rng, (rows, d), dt)
    resid = _rnd(rng, (rows, d), dt)
    tx, tg, tb, tdy, tres = (to_dev(a, dt) for a in (x, g, b, dy, resid))
    y = torch.zeros_like(tx)
    dx = torch.zeros_like(tx)
    stats = torch.zeros((2, rows), dtype=F32, device=DEV)
    dg = torch.full((d,), 1.0, dtype=F32, device=DEV)
    db = torch.full((d,), 1.0, dtype=F32, device=DEV)
    partial = torch.zeros(ds.ds_norm_bwd_scratch_floats(rows, d), dtype=F32, device=DEV)
    ds.ds_norm_fwd(tx, tg, None if rms else tb, y, stats, rms=rms)
    ds.ds_norm_bwd(tdy, tx, tg, stats, tres, dx, dg, None if rms else db, partial, rms=rms, accumulate=True)
    torch.cuda.synchronize()
    X, G, DY = x.astype(np.float64), g.astype(np.float64), dy.astype(np.float64)
    if rms:
        ref_y, cache = ost.rmsnorm_fwd(X, G)
        ref_dx, ref_dg = ost.rmsnorm_bwd(DY, cache, G)
        ref_db = None
    else:
        ref_y, cache = ost.layernorm_fwd(X, G, b.astype(np.float64))
        ref_dx, ref_dg, ref_db = ost.layernorm_bwd(DY, cache, G)
    tol = 6e-3 if dt == BF else 2e-5
    assert both_err(to_np(y), ref_y) <= tol
    assert both_err(to_np(dx), ref_dx + resid) <= tol
    assert both_err(to_np(dg), ref_dg + 1.0) <= 1e-4
    if not rms:
        assert both_err(to_np(db), ref_db + 1.0) <= 1e-4


@pytest.mark.parametrize("dt", [F32, BF])
def test_colsum(dt):
    rng = np.random.default_rng(7)
    rows, n = 5000 + 7, 1536
    x = _rnd(rng, (rows, n), dt)
    tx = to_dev(x, dt)
    out = torch.full((n,), 2.0, dtype=F32, device=DEV)
    partial = torch.zeros(ds.ds_norm_bwd_scratch_floats(rows, n), dtype=F32, device=DEV)
    ds.ds_colsum(tx, out, partial, accumulate=True)
    ds.ds_colsum(tx, out, partial, accumulate=False)
    torch.cuda.synchronize()
    assert both_err(to_np(out), x.astype(np.float64).sum(axis=0)) <= 1e-5


def test_pack_unpack_roundtrip():
    lens = np.array([5, 3, 9, 3, 7, 2], dtype=np.int32)
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=10 ** 6, lin=1), 18, 2)
    d = 16
    canon = torch.arange(int(lens.sum()) * d, dtype=F32, device=DEV).reshape(-1, d).contiguous()
    stream = torch.full((lo.total_rows, d), float("nan"), dtype=F32, device=DEV)
    ds.ds_pack(lo, canon, stream)
    host = stream.cpu().numpy()
    off = np.concatenate([[0], np.cumsum(lens)])
    valid = np.zeros(lo.total_rows, bool)
    for s in range(lo.n_seq):
        i = int(lo.perm[s])
        r = int(lo.seq_row[s])
        np.testing.assert_array_equal(host[r:r + lens[i]], canon.cpu().numpy()[off[i]:off[i + 1]])
        valid[r:r + lens[i]] = True
    assert np.all(host[~valid] == 0)
    back = torch.zeros_like(canon)
    ds.ds_unpack(lo, stream, back)
    assert torch.equal(back, canon)


# ---- the direct-to-LDS matrix-core kernel (NT / TN forms) at operator level, with and without the split-K workspace

def _ws(floats):
    return torch.zeros(floats, dtype=F32, device=DEV)


@pytest.mark.parametrize("use_ws", [False, True])
@pytest.mark.parametrize("M,N,K", [(700, 256, 128), (1037, 512, 1024), (5157, 3328, 1024)])
def test_gemm_nt_epilogues(use_ws, M, N, K):
    """C = A B^T with B given as [N, K] (forward with transposed weights, input gradients): every epilogue, ragged M,
    launches with fewer tiles than compute units (all tiles split over K when a workspace is given) and with more
    (whole rounds unsplit, the remaining tiles split)."""
    rng = np.random.default_rng(12)
    A, B = _rnd(rng, (M, K), BF), _rnd(rng, (N, K), BF, 0.1)
    bias, R, R2 = _rnd(rng, (N,), BF), _rnd(rng, (M, N), BF), _rnd(rng, (M, N), BF)
    valid = np.where(rng.random(M) < 0.8, 1, -1).astype(np.int32)
    acc = A.astype(np.float64) @ B.astype(np.float64).T
    dA, dB, db, dR, dR2 = (to_dev(x, BF) for x in (A, B, bias, R, R2))
    dvalid = torch.from_numpy(valid).to(DEV)
    ws = _ws(40 * 256 * 256) if use_ws else None
    tol = 6e-3

    def run(epi, **kw):
        c = torch.zeros((M, N), dtype=BF, device=DEV)
        c2 = torch.zeros((M, N), dtype=BF, device=DEV)
        ds.ds_gemm(dA, dB, c, M, N, K, trans_b=True, epilogue=epi, C2=c2, workspace=ws, **kw)
        torch.cuda.synchronize()
        return to_np(c), to_np(c2)

    c, _ = run(ds.DS_EPI_NONE)
    assert both_err(c, acc) <= tol
    c, _ = run(ds.DS_EPI_NONE, bias=db)
    assert both_err(c, acc + bias) <= tol
    z, a = run(ds.DS_EPI_GELU, bias=db)
    assert both_err(z, acc + bias) <= tol and both_err(a, ost.gelu(acc + bias)) <= tol
    c, _ = run(ds.DS_EPI_RESID, bias=db, R=dR, row_valid=dvalid)
    assert both_err(c, (acc + bias + R) * (valid[:, None] >= 0)) <= tol and np.all(c[valid < 0] == 0)
    c, _ = run(ds.DS_EPI_DGELU, R=dR)
    assert both_err(c, acc * ost.gelu_grad(R.astype(np.float64))) <= tol
    gd, a = run(ds.DS_EPI_GELU_D, bias=db)                # derivative kept instead of the pre-activation
    assert both_err(gd, ost.gelu_grad(acc + bias)) <= tol and both_err(a, ost.gelu(acc + bias)) <= tol
    c, _ = run(ds.DS_EPI_MULR, R=dR)
    assert both_err(c, acc * R) <= tol
    zu, h = run(ds.DS_EPI_GATE, R=dR)
    assert both_err(zu, acc) <= tol and both_err(h, ost.gelu(R.astype(np.float64)) * acc) <= tol
    g1, g2 = run(ds.DS_EPI_DGATE, R=dR, R2=dR2)
    assert both_err(g1, acc * R2 * ost.gelu_grad(R.astype(np.float64))) <= tol
    assert both_err(g2, acc * ost.gelu(R.astype(np.float64))) <= tol


@pytest.mark.parametrize("M,N,K", [(512, 768, 2085), (256, 256, 4100), (2048, 2048, 1031)])
def test_gemm_weight_gradient_split_over_the_contraction(M, N, K):
    """dW = X^T dY with a workspace: the contraction is cut into ranges (ragged last tile), partial sums added by the
    second kernel; overwrite and accumulate; same result as the unsplit launch up to summation order."""
    rng = np.random.default_rng(13)
    X, dY = _rnd(rng, (K, M), BF), _rnd(rng, (K, N), BF)
    ref = X.astype(np.float64).T @ dY.astype(np.float64)
    dX, ddY = to_dev(X, BF), to_dev(dY, BF)
    ws = _ws(4 * M * N + 4096)
    Cd = torch.full((M, N), 3.0, dtype=F32, device=DEV)
    ds.ds_gemm(dX, ddY, Cd, M, N, K, trans_a=True, epilogue=ds.DS_EPI_ACC32, accumulate=False, workspace=ws)
    torch.cuda.synchronize()
    assert both_err(to_np(Cd), ref) <= 1e-5
    ds.ds_gemm(dX, ddY, Cd, M, N, K, trans_a=True, epilogue=ds.DS_EPI_ACC32, accumulate=True, workspace=ws)
    torch.cuda.synchronize()
    assert both_err(to_np(Cd), 2 * ref) <= 1e-5
    plain = torch.zeros((M, N), dtype=F32, device=DEV)
    ds.ds_gemm(dX, ddY, plain, M, N, K, trans_a=True, epilogue=ds.DS_EPI_ACC32, accumulate=False)
    torch.cuda.synchronize()
    assert both_err(to_np(plain), ref) <= 1e-5


@pytest.mark.parametrize("use_ws", [False, True])
def test_gemm_nt_persistent_form(use_ws):
    """A launch with at least two unsplit tiles per compute unit takes the persistent form of the NT kernel (resident
    work-groups drawing tiles from per-XCD counters; with a workspace the last tiles are split pieces behind them):
    every tile against the reference, ragged M, several epilogues; again on another stream and a third time, bit for
    bit the same (the counters a launch leaves behind are those the next one starts from)."""
    rng = np.random.default_rng(21)
    M, N, K = 256 * 40 + 57, 3328, 512                     # 41 x 13 = 533 tiles
    A, B = _rnd(rng, (M, K), BF), _rnd(rng, (N, K), BF, 0.1)
    bias, R = _rnd(rng, (N,), BF), _rnd(rng, (M, N), BF)
    valid = np.where(rng.random(M) < 0.9, 1, -1).astype(np.int32)
    acc = A.astype(np.float64) @ B.astype(np.float64).T
    dA, dB, db, dR = (to_dev(x, BF) for x in (A, B, bias, R))
    dvalid = torch.from_numpy(valid).to(DEV)
    ws = _ws(64 * 256 * 256) if use_ws else None
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    tol = 6e-3

    def run(epi, stream=None, **kw):
        c = torch.zeros((M, N), dtype=BF, device=DEV)
        c2 = torch.zeros((M, N), dtype=BF, device=DEV)
        ds.ds_gemm(dA, dB, c, M, N, K, trans_b=True, epilogue=epi, C2=c2, workspace=ws, stream=stream, **kw)
        torch.cuda.synchronize()
        return to_np(c), to_np(c2)

    for epi, kw, want, want2 in [
            (ds.DS_EPI_NONE, dict(bias=db), acc + bias, None),
            (ds.DS_EPI_RESID, dict(bias=db, R=dR, row_valid=dvalid), (acc + bias + R) * (valid[:, None] >= 0), None),
            (ds.DS_EPI_GELU_D, dict(bias=db), ost.gelu_grad(acc + bias), ost.gelu(acc + bias)),
            (ds.DS_EPI_MULR, dict(R=dR), acc * R, None)]:
        c, c2 = run(epi, **kw)
        assert both_err(c, want) <= tol
        if want2 is not None:
            assert both_err(c2, want2) <= tol
        for stream in (side.cuda_stream, None):
            d, d2 = run(epi, stream=stream, **kw)
            assert np.array_equal(c, d)
            if want2 is not None:
                assert np.array_equal(c2, d2)


def test_mfma_probe_runs_and_is_deterministic():
    """The measurement aid: the loop really runs (sums differ from zero on random operands, are zero on zeros) and
    gives the same sums every time."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    ops = torch.randn(24 * 512 * 8, device=DEV, generator=gen).to(BF)
    sink = torch.zeros(2 * 512, dtype=F32, device=DEV)
    ds.ds_mfma_probe(ops, sink, 2, 3)
    torch.cuda.synchronize()
    first = to_np(sink)
    assert np.all(np.isfinite(first)) and np.count_nonzero(first) > 900
    assert np.array_equal(first[:512], first[512:])             # every work-group computes the same
    ds.ds_mfma_probe(ops, sink, 2, 3)
    torch.cuda.synchronize()
    assert np.array_equal(first, to_np(sink))
    ds.ds_mfma_probe(torch.zeros_like(ops), sink, 2, 3)
    torch.cuda.synchronize()
    assert np.count_nonzero(to_np(sink)) == 0
    with pytest.raises(ds.DsError):
        ds.ds_mfma_probe(ops, sink, 0, 3)
