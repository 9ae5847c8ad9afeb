"""ctypes binding of libdynastage.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/dynastage.h); all
compute happens in the library.  torch tensors are used as device memory: their data_ptr() is
what crosses the boundary.  Loading fails loudly when the library has not been built
(`python -m paper_2311_10418_amd.build`); there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdynastage.so")

DS_OK, DS_EINVAL, DS_EINFEASIBLE, DS_ENOMEM, DS_EOVERFLOW, DS_EHIP, DS_ELAYOUT, DS_ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7
DS_COST_POLY_GPT, DS_COST_POLY_T5, DS_COST_TABLE = 0, 1, 2
DS_MODEL_GPT, DS_MODEL_T5 = 0, 1
DS_DTYPE_F32, DS_DTYPE_BF16 = 0, 1
DS_EPI_NONE, DS_EPI_GELU, DS_EPI_RESID, DS_EPI_DGELU, DS_EPI_ACC32, DS_EPI_GATE, DS_EPI_DGATE, DS_EPI_GELU_D, DS_EPI_MULR = range(9)

PROF_KINDS = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "norm", "colsum", "other", "transpose")

_STATUS_NAMES = {0: "DS_OK", -1: "DS_EINVAL", -2: "DS_EINFEASIBLE", -3: "DS_ENOMEM", -4: "DS_EOVERFLOW",
                 -5: "DS_EHIP", -6: "DS_ELAYOUT", -7: "DS_ELIMIT"}

EXPORTS = ["dp_plan", "dp_plan_sampled", "dp_plan_replicas", "ds_plan_recompute", "ds_assign_replicas", "ds_cost_table_build", "ds_schedule_adaptive",
           "ds_schedule_1f1b", "ds_schedule_simulate", "ds_comm_plan", "ds_layout_from_cuts", "ds_layout_token_based", "ds_layout_packed", "ds_layout_get", "ds_layout_free",
           "ds_stage_create", "ds_stage_destroy", "ds_stage_workspace_bytes", "ds_stage_workspace_need", "stage_fwd_bwd",
           "ds_stage_last_launch_count", "ds_stage_weights_unchanged", "ds_stage_profile_enable", "ds_stage_profile_read", "ds_pack", "ds_unpack", "ds_gemm", "ds_gemm_ws", "ds_attention_fwd",
           "ds_attention_bwd", "ds_attention_scratch_bytes", "ds_norm_fwd", "ds_norm_bwd", "ds_norm_bwd_scratch_floats", "ds_colsum", "ds_colsum_static",
           "ds_mfma_probe", "ds_version"]


class DsError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("%s returned %s (%d)" % (where, _STATUS_NAMES.get(code, "?"), code))
        self.code = code


class ds_cost_model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("fixed", C.c_int64), ("lin", C.c_int64),
                ("table", C.c_void_p), ("tb", C.c_int32), ("tl", C.c_int32)]


class ds_recompute_scheme(C.Structure):
    _fields_ = [("cm", ds_cost_model), ("act_per_row", C.c_int64), ("fwd_num", C.c_int64), ("fwd_den", C.c_int64)]


_I32P = C.POINTER(C.c_int32)


class ds_layout_view(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_mb", C.c_int32),
                ("total_rows", C.c_int32), ("total_rows_tgt", C.c_int32),
                ("total_tokens", C.c_int64), ("total_tokens_tgt", C.c_int64),
                ("objective", C.c_int64), ("t_max", C.c_int64),
                ("perm", _I32P), ("mb_start", _I32P), ("mb_count", _I32P), ("mb_lpad", _I32P), ("mb_ltgt", _I32P),
                ("mb_cost", C.POINTER(C.c_int64)), ("mb_row", _I32P), ("mb_nrows", _I32P), ("mb_row_tgt", _I32P), ("mb_nrows_tgt", _I32P),
                ("seq_row", _I32P), ("seq_len", _I32P), ("seq_row_tgt", _I32P), ("seq_len_tgt", _I32P)]


class ds_stage_config(C.Structure):
    _fields_ = [("model", C.c_int32), ("dtype", C.c_int32), ("n_layers", C.c_int32), ("n_dec_layers", C.c_int32),
                ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("max_rows", C.c_int32), ("max_rows_tgt", C.c_int32), ("max_seqs", C.c_int32), ("recompute", C.c_int32)]


DS_RECOMPUTE_NONE, DS_RECOMPUTE_FULL = 0, 1


GPT_KEYS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")
T5_ENC_KEYS = ("ln1_g", "w_qkv", "w_o", "ln2_g", "w_g", "w_u", "w_2")
T5_DEC_KEYS = ("ln1_g", "w_qkv", "w_o", "lnc_g", "w_cq", "w_ckv", "w_co", "ln2_g", "w_g", "w_u", "w_2")


class ds_gpt_layer(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in GPT_KEYS]


class ds_t5_enc_layer(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in T5_ENC_KEYS]


class ds_t5_dec_layer(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in T5_DEC_KEYS]


class ds_stage_io(C.Structure):
    _fields_ = [("act_in", C.c_void_p), ("act_in_tgt", C.c_void_p), ("grad_out", C.c_void_p),
                ("act_out", C.c_void_p), ("grad_in", C.c_void_p), ("grad_in_tgt", C.c_void_p)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdynastage.so is missing: run `python -m paper_2311_10418_amd.build` "
                               "(there is no fallback implementation)")
        try:
            # PyTorch ships its own HIP runtime; loading it first makes this library bind to that copy, so the
            # process holds ONE runtime (with two, allocations from the second one fail)
            import torch  # noqa: F401
        except ImportError:
            pass
        _lib = C.CDLL(LIB_PATH)
        _lib.ds_version.restype = C.c_char_p
        _lib.ds_stage_workspace_bytes.restype = C.c_int64
        _lib.ds_stage_workspace_need.restype = C.c_int64
        _lib.ds_norm_bwd_scratch_floats.restype = C.c_int64
        _lib.ds_attention_scratch_bytes.restype = C.c_int64
        _lib.ds_layout_free.restype = None
        _lib.ds_stage_destroy.restype = None
    return _lib


def _check(code, where):
    if code != DS_OK:
        raise DsError(code, where)


def _np_i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _hp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dp(t):
    """Device (or host) pointer of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_contiguous(), "tensors crossing the boundary must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return DS_DTYPE_BF16
    if t.dtype == torch.float32:
        return DS_DTYPE_F32
    raise TypeError("unsupported dtype %s" % t.dtype)


def make_cost_model(kind=DS_COST_POLY_GPT, fixed=0, lin=2048, table=None):
    cm = ds_cost_model()
    cm.kind, cm.fixed, cm.lin = kind, fixed, lin
    cm._keep = None
    if table is not None:
        tab = np.ascontiguousarray(table, dtype=np.int64)
        cm._keep = tab
        cm.table = tab.ctypes.data
        cm.tb, cm.tl = tab.shape
    return cm


def ds_cost_table_build(b_grid, l_grid, t, tb, tl, scale=1.0, inf_cost=1 << 50):
    """int64 table [tb, tl] for make_cost_model(kind=DS_COST_TABLE, table=...) from profiled times t[nb, nl]."""
    bg, lg = _np_i32(b_grid), _np_i32(l_grid)
    tt = np.ascontiguousarray(t, dtype=np.float64)
    if tt.shape != (bg.shape[0], lg.shape[0]):
        raise ValueError("t must have shape [len(b_grid), len(l_grid)]")
    out = np.empty((tb, tl), dtype=np.int64)
    rc = lib().ds_cost_table_build(_hp(bg), C.c_int32(bg.shape[0]), _hp(lg), C.c_int32(lg.shape[0]),
                                   tt.ctypes.data_as(C.c_void_p), C.c_double(scale), C.c_int32(tb), C.c_int32(tl),
                                   C.c_int64(inf_cost), out.ctypes.data_as(C.c_void_p))
    _check(rc, "ds_cost_table_build")
    return out


class Layout:
    """Owns a ds_layout*; exposes the view's arrays as numpy copies."""

    def __init__(self, handle):
        self.handle = handle
        v = ds_layout_view()
        _check(lib().ds_layout_get(handle, C.byref(v)), "ds_layout_get")
        self.n_seq, self.n_mb = v.n_seq, v.n_mb
        self.total_rows, self.total_rows_tgt = v.total_rows, v.total_rows_tgt
        self.total_tokens, self.total_tokens_tgt = v.total_tokens, v.total_tokens_tgt
        self.objective, self.t_max = v.objective, v.t_max

        def arr(p, n):
            return None if not p else np.ctypeslib.as_array(p, shape=(n,)).copy()

        for name in ("perm", "seq_row", "seq_len", "seq_row_tgt", "seq_len_tgt"):
            setattr(self, name, arr(getattr(v, name), v.n_seq))
        for name in ("mb_start", "mb_count", "mb_lpad", "mb_ltgt", "mb_cost", "mb_row", "mb_nrows", "mb_row_tgt", "mb_nrows_tgt"):
            setattr(self, name, arr(getattr(v, name), v.n_mb))

    @property
    def cuts(self):
        return np.concatenate([self.mb_start, [self.n_seq]]).astype(np.int32)

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ds_layout_free(self.handle)
            self.handle = None


def dp_plan(lengths, cost_model, mem_cap_tokens, num_stages, lengths_tgt=None):
    ln, lt = _np_i32(lengths), _np_i32(lengths_tgt)
    out = C.c_void_p()
    n = 0 if ln is None else int(ln.shape[0])
    rc = lib().dp_plan(_hp(ln), _hp(lt), C.c_int32(n), C.byref(cost_model) if cost_model is not None else None,
                       C.c_int64(mem_cap_tokens), C.c_int32(num_stages), C.byref(out))
    _check(rc, "dp_plan")
    return Layout(out)


def ds_plan_recompute(lengths, schemes, mem_limit, num_stages, lengths_tgt=None):
    """schemes: list of (cost_model, act_per_row, fwd_num, fwd_den).
    -> (chosen index, Layout of the chosen scheme, makespan int64[n_schemes], peak int64[n_schemes]); -1 marks an
    infeasible scheme."""
    ln, lt = _np_i32(lengths), _np_i32(lengths_tgt)
    n = 0 if ln is None else int(ln.shape[0])
    k = len(schemes)
    arr = (ds_recompute_scheme * max(k, 1))()
    keep = []
    for r, (cm, a, fn, fd) in enumerate(schemes):
        arr[r].cm.kind, arr[r].cm.fixed, arr[r].cm.lin = cm.kind, cm.fixed, cm.lin
        arr[r].cm.table, arr[r].cm.tb, arr[r].cm.tl = cm.table, cm.tb, cm.tl
        keep.append(cm)                                     # the table memory stays alive through the call
        arr[r].act_per_row, arr[r].fwd_num, arr[r].fwd_den = int(a), int(fn), int(fd)
    out = C.c_void_p()
    chosen = C.c_int32(-1)
    ms = np.zeros(max(k, 1), dtype=np.int64)
    pk = np.zeros(max(k, 1), dtype=np.int64)
    rc = lib().ds_plan_recompute(_hp(ln), _hp(lt), C.c_int32(n), arr if k else None, C.c_int32(k), C.c_int64(mem_limit),
                                 C.c_int32(num_stages), C.byref(chosen), C.byref(out), _hp(ms), _hp(pk))
    _check(rc, "ds_plan_recompute")
    return int(chosen.value), Layout(out), ms[:k], pk[:k]


def dp_plan_sampled(lengths, cost_model, mem_cap_tokens, num_stages, t_max_interval, lengths_tgt=None):
    ln, lt = _np_i32(lengths), _np_i32(lengths_tgt)
    out = C.c_void_p()
    n = 0 if ln is None else int(ln.shape[0])
    rc = lib().dp_plan_sampled(_hp(ln), _hp(lt), C.c_int32(n), C.byref(cost_model) if cost_model is not None else None,
                               C.c_int64(mem_cap_tokens), C.c_int32(num_stages), C.c_int64(t_max_interval), C.byref(out))
    _check(rc, "dp_plan_sampled")
    return Layout(out)


def dp_plan_replicas(lengths, cost_model, mem_cap_tokens, num_stages, n_replicas, lengths_tgt=None):
    """-> (Layout, replica_of_mb int32[n_mb], replica_time int64[n_replicas])."""
    ln, lt = _np_i32(lengths), _np_i32(lengths_tgt)
    out = C.c_void_p()
    n = 0 if ln is None else int(ln.shape[0])
    rep = np.zeros(max(n, 1), dtype=np.int32)
    sums = np.zeros(max(int(n_replicas), 1), dtype=np.int64)
    rc = lib().dp_plan_replicas(_hp(ln), _hp(lt), C.c_int32(n), C.byref(cost_model) if cost_model is not None else None,
                                C.c_int64(mem_cap_tokens), C.c_int32(num_stages), C.c_int32(n_replicas), C.byref(out),
                                rep.ctypes.data_as(C.c_void_p), sums.ctypes.data_as(C.c_void_p))
    _check(rc, "dp_plan_replicas")
    lay = Layout(out)
    return lay, rep[:lay.n_mb].copy(), sums


def ds_assign_replicas(times, n_replicas):
    """Karmarkar-Karp split of `times` into n_replicas sets -> (replica_of int32[n], replica_time int64[n_replicas])."""
    t = np.ascontiguousarray(times, dtype=np.int64)
    rep = np.zeros(max(t.shape[0], 1), dtype=np.int32)
    sums = np.zeros(max(int(n_replicas), 1), dtype=np.int64)
    rc = lib().ds_assign_replicas(t.ctypes.data_as(C.c_void_p), C.c_int32(t.shape[0]), C.c_int32(n_replicas),
                                  rep.ctypes.data_as(C.c_void_p), sums.ctypes.data_as(C.c_void_p))
    _check(rc, "ds_assign_replicas")
    return rep[:t.shape[0]].copy(), sums


def _i64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.int64)
    if shape is not None and a.shape != shape:
        raise ValueError("expected an int64 array of shape %s, got %s" % (shape, a.shape))
    return a


def _vp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def ds_schedule_adaptive(act, limit):
    """act [M, C], limit [C] -> (order_mb [C, 2M], order_kind [C, 2M], cycles)."""
    act = _i64(act)
    M, Cn = act.shape
    limit = _i64(limit, (Cn,))
    omb, okind = np.zeros((Cn, 2 * M), np.int32), np.zeros((Cn, 2 * M), np.int32)
    cyc = C.c_int32(0)
    _check(lib().ds_schedule_adaptive(C.c_int32(Cn), C.c_int32(M), _vp(act), _vp(limit), _vp(omb), _vp(okind), C.byref(cyc)),
           "ds_schedule_adaptive")
    return omb, okind, cyc.value


def ds_schedule_1f1b(n_stages, n_mb):
    omb, okind = np.zeros((n_stages, 2 * n_mb), np.int32), np.zeros((n_stages, 2 * n_mb), np.int32)
    _check(lib().ds_schedule_1f1b(C.c_int32(n_stages), C.c_int32(n_mb), _vp(omb), _vp(okind)), "ds_schedule_1f1b")
    return omb, okind


def ds_schedule_simulate(order_mb, order_kind, t_fwd, t_bwd, act=None):
    """-> dict(makespan, idle [C], peak [C] or None, start [C, 2M], end [C, 2M])."""
    omb = np.ascontiguousarray(order_mb, dtype=np.int32)
    okind = np.ascontiguousarray(order_kind, dtype=np.int32)
    Cn, M2 = omb.shape
    M = M2 // 2
    tf, tb = _i64(t_fwd, (M, Cn)), _i64(t_bwd, (M, Cn))
    a = None if act is None else _i64(act, (M, Cn))
    mk = C.c_int64(0)
    idle, peak = np.zeros(Cn, np.int64), (np.zeros(Cn, np.int64) if a is not None else None)
    st, en = np.zeros((Cn, M2), np.int64), np.zeros((Cn, M2), np.int64)
    _check(lib().ds_schedule_simulate(C.c_int32(Cn), C.c_int32(M), _vp(omb), _vp(okind), _vp(tf), _vp(tb), _vp(a), C.byref(mk),
                                      _vp(idle), _vp(peak), _vp(st), _vp(en)), "ds_schedule_simulate")
    return {"makespan": mk.value, "idle": idle, "peak": peak, "start": st, "end": en}


def ds_comm_plan(order_mb, order_kind, t_fwd, t_bwd):
    """-> list over stages of [(DS_INSTR_* code, micro-batch), ...]."""
    omb = np.ascontiguousarray(order_mb, dtype=np.int32)
    okind = np.ascontiguousarray(order_kind, dtype=np.int32)
    Cn, M2 = omb.shape
    M = M2 // 2
    tf, tb = _i64(t_fwd, (M, Cn)), _i64(t_bwd, (M, Cn))
    code, mb, ln = np.zeros((Cn, 8 * M), np.int32), np.zeros((Cn, 8 * M), np.int32), np.zeros(Cn, np.int32)
    _check(lib().ds_comm_plan(C.c_int32(Cn), C.c_int32(M), _vp(omb), _vp(okind), _vp(tf), _vp(tb), _vp(code), _vp(mb), _vp(ln)),
           "ds_comm_plan")
    return [[(int(code[j, k]), int(mb[j, k])) for k in range(ln[j])] for j in range(Cn)]


def ds_layout_from_cuts(lengths, cuts, perm=None, lengths_tgt=None, pad_to=0, pad_to_tgt=0, cost_model=None, num_stages=1):
    ln, lt, pm, ct = _np_i32(lengths), _np_i32(lengths_tgt), _np_i32(perm), _np_i32(cuts)
    out = C.c_void_p()
    rc = lib().ds_layout_from_cuts(_hp(ln), _hp(lt), C.c_int32(len(ln)), _hp(pm), _hp(ct), C.c_int32(len(ct) - 1),
                                   C.c_int32(pad_to), C.c_int32(pad_to_tgt),
                                   C.byref(cost_model) if cost_model is not None else None,
                                   C.c_int32(num_stages), C.byref(out))
    _check(rc, "ds_layout_from_cuts")
    return Layout(out)


def ds_layout_token_based(lengths, token_budget, lengths_tgt=None, cost_model=None, num_stages=1):
    ln, lt = _np_i32(lengths), _np_i32(lengths_tgt)
    out = C.c_void_p()
    rc = lib().ds_layout_token_based(_hp(ln), _hp(lt), C.c_int32(len(ln)), C.c_int64(token_budget),
                                     C.byref(cost_model) if cost_model is not None else None,
                                     C.c_int32(num_stages), C.byref(out))
    _check(rc, "ds_layout_token_based")
    return Layout(out)


def ds_layout_packed(lengths, row_len, rows_per_mb):
    ln = _np_i32(lengths)
    out = C.c_void_p()
    rc = lib().ds_layout_packed(_hp(ln), C.c_int32(len(ln)), C.c_int32(row_len), C.c_int32(rows_per_mb), C.byref(out))
    _check(rc, "ds_layout_packed")
    return Layout(out)


def _layer_array(struct, keys, layers):
    arr = (struct * len(layers))()
    for i, layer in enumerate(layers):
        for k in keys:
            setattr(arr[i], k, layer[k].data_ptr())
    return arr


def ds_stage_workspace_need(model, dtype, n_layers, d_model, n_heads, d_ff, max_rows, max_seqs, n_dec_layers=0, max_rows_tgt=0,
                            recompute=DS_RECOMPUTE_NONE):
    """Bytes of device workspace a Stage with this configuration allocates (host only; no GPU needed)."""
    cfg = ds_stage_config(model, dtype, n_layers, n_dec_layers, d_model, n_heads, d_ff, max_rows, max_rows_tgt, max_seqs, recompute)
    need = lib().ds_stage_workspace_need(C.byref(cfg))
    if need < 0:
        raise DsError(-1, "ds_stage_workspace_need")
    return int(need)


class Stage:
    """Owns a ds_stage* (device workspace)."""

    def __init__(self, model, dtype, n_layers, d_model, n_heads, d_ff, max_rows, max_seqs, n_dec_layers=0, max_rows_tgt=0,
                 recompute=DS_RECOMPUTE_NONE):
        cfg = ds_stage_config(model, dtype, n_layers, n_dec_layers, d_model, n_heads, d_ff, max_rows, max_rows_tgt, max_seqs,
                              recompute)
        self.cfg = cfg
        h = C.c_void_p()
        _check(lib().ds_stage_create(C.byref(cfg), C.byref(h)), "ds_stage_create")
        self.handle = h

    def workspace_bytes(self):
        return lib().ds_stage_workspace_bytes(self.handle)

    def last_launch_count(self):
        return lib().ds_stage_last_launch_count(self.handle)

    def weights_unchanged(self, unchanged=True):
        """Promise that the following calls get the weights of the previous call, contents included."""
        _check(lib().ds_stage_weights_unchanged(self.handle, C.c_int32(int(unchanged))), "ds_stage_weights_unchanged")

    def profile_enable(self, on=True):
        _check(lib().ds_stage_profile_enable(self.handle, C.c_int32(int(on))), "ds_stage_profile_enable")

    def profile_read(self):
        """-> dict kind -> (milliseconds, groups) summed since the last read."""
        ms = (C.c_float * len(PROF_KINDS))()
        cnt = (C.c_int32 * len(PROF_KINDS))()
        _check(lib().ds_stage_profile_read(self.handle, ms, cnt), "ds_stage_profile_read")
        return {k: (ms[i], cnt[i]) for i, k in enumerate(PROF_KINDS)}

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ds_stage_destroy(self.handle)
            self.handle = None

    __del__ = close


def stage_fwd_bwd(stage, layout, weights, act_in, grad_out, act_out, grad_in, grads, accumulate=False, stream=None,
                  weights_dec=None, grads_dec=None, act_in_tgt=None, grad_in_tgt=None):
    """weights / grads: list (one dict per layer) of torch tensors keyed as GPT_KEYS (or T5_ENC_KEYS; then
    weights_dec / grads_dec keyed as T5_DEC_KEYS).  All tensors already on the device."""
    if stage.cfg.model == DS_MODEL_GPT:
        w = _layer_array(ds_gpt_layer, GPT_KEYS, weights)
        g = _layer_array(ds_gpt_layer, GPT_KEYS, grads)
        wd = gd = None
    else:
        w = _layer_array(ds_t5_enc_layer, T5_ENC_KEYS, weights)
        g = _layer_array(ds_t5_enc_layer, T5_ENC_KEYS, grads)
        wd = _layer_array(ds_t5_dec_layer, T5_DEC_KEYS, weights_dec)
        gd = _layer_array(ds_t5_dec_layer, T5_DEC_KEYS, grads_dec)
    # the kernels address layout.total_rows rows of every activation tensor: refuse shorter ones here, where
    # the shapes are still known (the C ABI sees plain pointers)
    for name, t, rows in (("act_in", act_in, layout.total_rows), ("grad_out", grad_out, None), ("act_out", act_out, None),
                          ("grad_in", grad_in, layout.total_rows), ("act_in_tgt", act_in_tgt, layout.total_rows_tgt),
                          ("grad_in_tgt", grad_in_tgt, layout.total_rows_tgt)):
        if t is None:
            continue
        if rows is None:
            rows = layout.total_rows_tgt if stage.cfg.model != DS_MODEL_GPT else layout.total_rows
        if t.dim() != 2 or t.shape[0] < rows or t.shape[1] != stage.cfg.d_model or not t.is_contiguous():
            raise ValueError("%s must be a contiguous [>= %d, %d] tensor, got %s" % (name, rows, stage.cfg.d_model, tuple(t.shape)))
    io = ds_stage_io()
    io.act_in = act_in.data_ptr()
    io.act_in_tgt = act_in_tgt.data_ptr() if act_in_tgt is not None else None
    io.grad_out = grad_out.data_ptr()
    io.act_out = act_out.data_ptr()
    io.grad_in = grad_in.data_ptr()
    io.grad_in_tgt = grad_in_tgt.data_ptr() if grad_in_tgt is not None else None
    rc = lib().stage_fwd_bwd(stage.handle, layout.handle, w, wd, C.byref(io), g, gd,
                             C.c_int32(1 if accumulate else 0), _stream(stream))
    _check(rc, "stage_fwd_bwd")


def ds_pack(layout, canonical, stream_rows, which=0, stream=None):
    rc = lib().ds_pack(layout.handle, C.c_int32(which), C.c_int32(_dtype_code(canonical)), C.c_int32(canonical.shape[1]),
                       _dp(canonical), _dp(stream_rows), _stream(stream))
    _check(rc, "ds_pack")


def ds_unpack(layout, stream_rows, canonical, which=0, stream=None):
    rc = lib().ds_unpack(layout.handle, C.c_int32(which), C.c_int32(_dtype_code(canonical)), C.c_int32(canonical.shape[1]),
                         _dp(stream_rows), _dp(canonical), _stream(stream))
    _check(rc, "ds_unpack")


def ds_gemm(A, B, Cout, M, N, K, trans_a=False, trans_b=False, epilogue=DS_EPI_NONE, bias=None, R=None, R2=None, C2=None,
            row_valid=None, accumulate=False, force_generic=False, stream=None, workspace=None):
    """workspace: optional float32 device tensor that lets the matrix-core kernels split the contraction (ds_gemm_ws)."""
    args = [C.c_int32(_dtype_code(A)), C.c_int32(int(trans_a)), C.c_int32(int(trans_b)),
            C.c_int32(M), C.c_int32(N), C.c_int32(K), _dp(A), _dp(B), _dp(Cout), C.c_int32(epilogue),
            _dp(bias), _dp(R), _dp(R2), _dp(C2), _dp(row_valid), C.c_int32(int(accumulate)),
            C.c_int32(int(force_generic))]
    if workspace is None:
        rc = lib().ds_gemm(*args, _stream(stream))
        _check(rc, "ds_gemm")
    else:
        rc = lib().ds_gemm_ws(*args, _dp(workspace), C.c_int64(workspace.numel()), _stream(stream))
        _check(rc, "ds_gemm_ws")


def ds_attention_fwd(q, k, v, o, lse, q_row, q_len, k_row, k_len, n_heads, head_dim, causal, max_q_len, max_k_len,
                     ldq, ldk, ldv, ldo, lse_stride, k_total_rows=None, scratch=None, force_generic=False, stream=None):
    """q, k, v may be views into one QKV tensor: pass data pointers via tensors created with narrow()/select or ints."""
    rc = lib().ds_attention_fwd(C.c_int32(_dtype_code(o)), C.c_int32(q_row.shape[0]), C.c_int32(n_heads),
                                C.c_int32(head_dim), C.c_int32(int(causal)), _dp(q_row), _dp(q_len), _dp(k_row), _dp(k_len),
                                C.c_int32(max_q_len), C.c_int32(max_k_len), _dp(q), C.c_int32(ldq), _dp(k), C.c_int32(ldk),
                                _dp(v), C.c_int32(ldv), _dp(o), C.c_int32(ldo), _dp(lse), C.c_int32(lse_stride),
                                C.c_int32(k_total_rows if k_total_rows is not None else lse_stride), _dp(scratch),
                                C.c_int64(scratch.numel() * scratch.element_size() if scratch is not None else 0),
                                C.c_int32(int(force_generic)), _stream(stream))
    _check(rc, "ds_attention_fwd")


def ds_attention_scratch_bytes(n_heads, head_dim, q_total_rows, k_total_rows, n_seq):
    return lib().ds_attention_scratch_bytes(C.c_int32(n_heads), C.c_int32(head_dim), C.c_int32(q_total_rows),
                                            C.c_int32(k_total_rows), C.c_int32(n_seq))


def ds_attention_bwd(q, k, v, o, d_o, lse, delta, dq, dk, dv, q_row, q_len, k_row, k_len, n_heads, head_dim, causal,
                     max_q_len, max_k_len, ldq, ldk, ldv, ldo, lse_stride, k_total_rows=None, scratch=None,
                     force_generic=False, stream=None):
    rc = lib().ds_attention_bwd(C.c_int32(_dtype_code(o)), C.c_int32(q_row.shape[0]), C.c_int32(n_heads),
                                C.c_int32(head_dim), C.c_int32(int(causal)), _dp(q_row), _dp(q_len), _dp(k_row), _dp(k_len),
                                C.c_int32(max_q_len), C.c_int32(max_k_len), _dp(q), C.c_int32(ldq), _dp(k), C.c_int32(ldk),
                                _dp(v), C.c_int32(ldv), _dp(o), _dp(d_o), C.c_int32(ldo), _dp(lse), _dp(delta),
                                C.c_int32(lse_stride), _dp(dq), _dp(dk), _dp(dv),
                                C.c_int32(k_total_rows if k_total_rows is not None else lse_stride), _dp(scratch),
                                C.c_int64(scratch.numel() * scratch.element_size() if scratch is not None else 0),
                                C.c_int32(int(force_generic)), _stream(stream))
    _check(rc, "ds_attention_bwd")


def ds_norm_fwd(x, g, b, y, stats, rms=False, stream=None):
    rows, d = x.shape
    rc = lib().ds_norm_fwd(C.c_int32(_dtype_code(x)), C.c_int32(int(rms)), C.c_int32(rows), C.c_int32(d), _dp(x), _dp(g),
                           _dp(b), _dp(y), _dp(stats), _stream(stream))
    _check(rc, "ds_norm_fwd")


def ds_norm_bwd_scratch_floats(rows, d):
    return lib().ds_norm_bwd_scratch_floats(C.c_int32(rows), C.c_int32(d))


def ds_norm_bwd(dy, x, g, stats, resid, dx, dg, db, partial, rms=False, accumulate=False, stream=None):
    rows, d = x.shape
    rc = lib().ds_norm_bwd(C.c_int32(_dtype_code(x)), C.c_int32(int(rms)), C.c_int32(rows), C.c_int32(d), _dp(dy), _dp(x),
                           _dp(g), _dp(stats), _dp(resid), _dp(dx), _dp(dg), _dp(db), _dp(partial),
                           C.c_int32(int(accumulate)), _stream(stream))
    _check(rc, "ds_norm_bwd")


def ds_mfma_probe(operands, sink, n_groups, iters, stream=None):
    rc = lib().ds_mfma_probe(_dp(operands), _dp(sink), C.c_int32(n_groups), C.c_int32(iters), _stream(stream))
    _check(rc, "ds_mfma_probe")


def ds_colsum(x, out, partial, accumulate=False, stream=None):
    rows, n = x.shape
    rc = lib().ds_colsum(C.c_int32(_dtype_code(x)), C.c_int32(rows), C.c_int32(n), _dp(x), _dp(out), _dp(partial),
                         C.c_int32(int(accumulate)), _stream(stream))
    _check(rc, "ds_colsum")


def ds_colsum_static(x, out, accumulate=False, stream=None, rows=None, n=None):
    """ds_colsum without a scratch argument and without any allocation (the partial sums live in the library's image)."""
    if rows is None:
        rows, n = x.shape
    rc = lib().ds_colsum_static(C.c_int32(_dtype_code(x)), C.c_int32(rows), C.c_int32(n), _dp(x), _dp(out),
                                C.c_int32(int(accumulate)), _stream(stream))
    _check(rc, "ds_colsum_static")


def ds_version():
    return lib().ds_version().decode()
