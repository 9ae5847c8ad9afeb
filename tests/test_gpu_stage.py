"""GPU parity of stage_fwd_bwd against the per-sequence float64 oracle, through the C ABI.

Bar: normwise relative error <= 1e-4 for fp32 and <= 2e-2 for bf16 storage, for the outputs and input
gradients of EVERY SEQUENCE on its own and for each weight-gradient tensor, each with the elementwise
companion bound of helpers.check; padding rows of the outputs exactly zero; results
independent of the micro-batch layout (DP plan, padded DP plan, fixed padding, packing,
single-sequence micro-batches), with NaN planted in every padding row of the inputs."""
import numpy as np
import pytest
import torch

from oracle import stage as ost
from paper_2311_10418_amd import binding as ds
from paper_2311_10418_amd import workload as wl
from helpers import check, check_seqs, rel_err, run_gpt_stage

pytestmark = pytest.mark.gpu

TOL = {ds.DS_DTYPE_F32: 1e-4, ds.DS_DTYPE_BF16: 2e-2}


def _small_case(bf16, n_seq=None, seed=0):
    cfg = dict(wl.CONFIGS["gpt_small_fp32"])
    lens, _ = wl.draw_lengths(cfg["lengths"], seed=seed)
    if n_seq:
        lens = lens[:n_seq]
    params = wl.draw_params(wl.GPT_KEYS, cfg["n_layers"], cfg["d_model"], cfg["d_ff"], seed=seed, bf16=bf16)
    xs = wl.draw_embedded_tokens(lens, cfg["d_model"], seed=seed, bf16=bf16)
    dys = wl.draw_rows(lens, cfg["d_model"], seed=seed, tag=5, bf16=bf16)
    return cfg, lens, params, xs, dys


_ORACLE_CACHE = {}


def _oracle(key, xs, dys, params, h):
    if key not in _ORACLE_CACHE:
        _ORACLE_CACHE[key] = ost.gpt_stage_fwd_bwd(xs, dys, params, h)
    return _ORACLE_CACHE[key]


def _compare(tag, got, ref, tol):
    outs, dxs, grads, pad_o, pad_dx = got
    r_outs, r_dxs, r_grads = ref
    # outputs and input gradients: every sequence on its own; weight gradients: every tensor; each normwise AND elementwise
    errs = {"act_out": check_seqs(outs, r_outs, tol, tag + " act_out"), "grad_in": check_seqs(dxs, r_dxs, tol, tag + " grad_in")}
    for li, layer in enumerate(r_grads):
        for k, v in layer.items():
            errs["L%d.%s" % (li, k)] = check(grads[li][k], v, tol, "%s L%d.%s" % (tag, li, k))
    worst = max(errs, key=errs.get)
    print(tag, "worst", worst, "%.3e" % errs[worst])
    assert pad_o.size == 0 or np.all(pad_o == 0), tag
    assert pad_dx.size == 0 or np.all(pad_dx == 0), tag
    return errs


def _layouts(lens, cap, c):
    n = len(lens)
    yield "dp", ds.dp_plan(lens, ds.make_cost_model(), cap, c)
    yield "dp_overhead", ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cap, c)
    yield "fixed_pad", ds.ds_layout_from_cuts(lens, list(range(0, n, 8)) + [n], pad_to=int(max(lens)))
    yield "packed", ds.ds_layout_packed(lens, int(max(lens)), 4)
    yield "singletons", ds.ds_layout_from_cuts(lens, list(range(n + 1)))


@pytest.mark.parametrize("dtype_code", [ds.DS_DTYPE_F32, ds.DS_DTYPE_BF16])
def test_small_gpt_stage_matches_oracle_on_every_layout(dtype_code):
    bf16 = dtype_code == ds.DS_DTYPE_BF16
    cfg, lens, params, xs, dys = _small_case(bf16)
    ref = _oracle(("small", bf16), xs, dys, params, cfg["n_heads"])
    for name, lo in _layouts(lens, cfg["cap"], cfg["num_stages"]):
        got = run_gpt_stage(lo, cfg, params, xs, dys, dtype_code)
        _compare("%s/%s rows=%d tokens=%d" % ("bf16" if bf16 else "f32", name, lo.total_rows, lo.total_tokens),
                 got, ref, TOL[dtype_code])


def test_weight_gradients_accumulate_across_calls():
    cfg, lens, params, xs, dys = _small_case(True, n_seq=12)
    ref = _oracle(("small12", True), xs, dys, params, cfg["n_heads"])
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cfg["cap"], cfg["num_stages"])
    stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["d_ff"],
                     max_rows=lo.total_rows + 100, max_seqs=64)
    from helpers import params_to_dev, zero_grads_like
    grads = zero_grads_like(params_to_dev(params, torch.bfloat16))
    for g in grads:
        for v in g.values():
            v.fill_(123.0)                       # overwritten by the first (non-accumulating) call
    run_gpt_stage(lo, cfg, params, xs, dys, ds.DS_DTYPE_BF16, stage=stage, grads=grads, accumulate=False)
    got = run_gpt_stage(lo, cfg, params, xs, dys, ds.DS_DTYPE_BF16, stage=stage, grads=grads, accumulate=True)
    for li, layer in enumerate(ref[2]):
        for k, v in layer.items():
            check(got[2][li][k], 2 * v, 2e-2, "accumulated L%d.%s" % (li, k))
    # same stage object, another layout right after: tables are re-bound
    lo2 = ds.ds_layout_from_cuts(lens, list(range(len(lens) + 1)))
    got2 = run_gpt_stage(lo2, cfg, params, xs, dys, ds.DS_DTYPE_BF16, stage=stage)
    _compare("rebind", got2, ref, 2e-2)
    stage.close()


def test_weight_copies_are_reused_only_under_the_callers_promise():
    """Micro-batches of one iteration run on the same weights: with the promise the transposed copies are made once."""
    from helpers import params_to_dev, stream_from_seqs, to_np
    cfg, lens, params, xs, dys = _small_case(True, n_seq=12)
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cfg["cap"], cfg["num_stages"])
    d = cfg["d_model"]
    stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, cfg["n_layers"], d, cfg["n_heads"], cfg["d_ff"],
                     max_rows=lo.total_rows, max_seqs=64)
    w = params_to_dev(params, torch.bfloat16)
    x = stream_from_seqs(xs, lo, d, torch.bfloat16, 0.0)
    dy = stream_from_seqs(dys, lo, d, torch.bfloat16, 0.0)

    def call():
        out, dx = torch.empty_like(x), torch.empty_like(x)
        g = [{k: torch.zeros(v.shape, dtype=torch.float32, device=x.device) for k, v in layer.items()} for layer in w]
        ds.stage_fwd_bwd(stage, lo, w, x, dy, out, dx, g)
        torch.cuda.synchronize()
        return to_np(out), to_np(dx), stage.last_launch_count()

    call()                                       # (the first call of a layout also builds the attention work lists)
    out0, dx0, n0 = call()
    stage.weights_unchanged(True)
    out1, dx1, n1 = call()                       # first call under the promise: same weights as before, copies reused
    assert n1 == n0 - 4 * cfg["n_layers"]
    assert np.array_equal(out0, out1) and np.array_equal(dx0, dx1)
    # an optimizer step: the promise is withdrawn, the new weights are seen
    stage.weights_unchanged(False)
    for layer in w:
        layer["w_2"].mul_(0.5)
    out2, _, n2 = call()
    assert n2 == n0 and not np.array_equal(out0, out2)
    # under the promise again, but with other weight tensors: the copies are made anew all the same
    stage.weights_unchanged(True)
    w = params_to_dev(params, torch.bfloat16)
    out3, dx3, n3 = call()
    assert n3 == n0 and np.array_equal(out0, out3) and np.array_equal(dx0, dx3)
    stage.close()


def test_layout_too_large_for_workspace_is_rejected():
    cfg, lens, params, xs, dys = _small_case(True, n_seq=6)
    lo = ds.ds_layout_from_cuts(lens, list(range(len(lens) + 1)))
    stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, 1, cfg["d_model"], cfg["n_heads"], cfg["d_ff"],
                     max_rows=lo.total_rows - 1, max_seqs=64)
    with pytest.raises(ds.DsError) as e:
        run_gpt_stage(lo, dict(cfg, n_layers=1), params[:1], xs, dys, ds.DS_DTYPE_BF16, stage=stage)
    assert e.value.code == ds.DS_ELAYOUT
    stage.close()


def test_stage_call_can_be_captured_in_a_graph_and_replays_identically():
    """With its layout already bound (one eager call), stage_fwd_bwd only enqueues kernels: it can be captured in a
    HIP graph; every replay, with eager work and synchronisation in between, reproduces the eager result bit for bit."""
    cfg, lens, params, xs, dys = _small_case(True, n_seq=12)
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cfg["cap"], cfg["num_stages"])
    from helpers import params_to_dev, stream_from_seqs, zero_grads_like
    d = cfg["d_model"]
    stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, cfg["n_layers"], d, cfg["n_heads"], cfg["d_ff"],
                     max_rows=lo.total_rows, max_seqs=lo.n_seq)
    w = params_to_dev(params, torch.bfloat16)
    grads = zero_grads_like(w)
    x = stream_from_seqs(xs, lo, d, torch.bfloat16, 0.0)
    dy = stream_from_seqs(dys, lo, d, torch.bfloat16, 0.0)
    out, dx = torch.empty_like(x), torch.empty_like(x)

    def call():
        ds.stage_fwd_bwd(stage, lo, w, x, dy, out, dx, grads, accumulate=False)

    def snapshot():
        return [out.clone(), dx.clone()] + [g[k].clone() for g in grads for k in g]

    for _ in range(2):
        call()
    torch.cuda.synchronize()
    ref = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    torch.cuda.synchronize()
    for _ in range(3):
        out.fill_(3.0)
        dx.fill_(3.0)
        for g in grads:
            for v in g.values():
                v.fill_(3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, snapshot()):
            assert torch.equal(a, b)
        call()                                   # eager work between replays
        torch.cuda.synchronize()
    del graph
    stage.close()


def test_back_to_back_calls_on_a_caller_stream_without_host_synchronisation():
    """The bias-gradient column sums run on a stream of the stage's own and are joined before a call returns control of
    the caller's stream: calls enqueued back to back on a stream of the caller's, with nothing in between, leave the same
    bits as one call followed by a synchronisation, and buffers the caller overwrites right behind a call are not read
    late."""
    cfg, lens, params, xs, dys = _small_case(True, n_seq=12)
    lo = ds.dp_plan(lens, ds.make_cost_model(fixed=2_000_000), cfg["cap"], cfg["num_stages"])
    from helpers import params_to_dev, stream_from_seqs, zero_grads_like
    d = cfg["d_model"]
    stage = ds.Stage(ds.DS_MODEL_GPT, ds.DS_DTYPE_BF16, cfg["n_layers"], d, cfg["n_heads"], cfg["d_ff"],
                     max_rows=lo.total_rows, max_seqs=lo.n_seq)
    w = params_to_dev(params, torch.bfloat16)
    grads = zero_grads_like(w)
    x = stream_from_seqs(xs, lo, d, torch.bfloat16, 0.0)
    dy = stream_from_seqs(dys, lo, d, torch.bfloat16, 0.0)
    out, dx = torch.empty_like(x), torch.empty_like(x)
    ds.stage_fwd_bwd(stage, lo, w, x, dy, out, dx, grads, accumulate=False)
    torch.cuda.synchronize()
    ref = [out.clone(), dx.clone()] + [g[k].clone() for g in grads for k in g]
    dy_copy = dy.clone()
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        for _ in range(4):
            ds.stage_fwd_bwd(stage, lo, w, x, dy, out, dx, grads, accumulate=False, stream=st.cuda_stream)
            dy.fill_(float("nan"))                  # the caller reuses its gradient buffer right behind the call ...
            dy.copy_(dy_copy)                       # ... and refills it for the next one, all in stream order
    torch.cuda.synchronize()
    for a, b in zip(ref, [out, dx] + [g[k] for g in grads for k in g]):
        assert torch.equal(a, b)
    stage.close()
