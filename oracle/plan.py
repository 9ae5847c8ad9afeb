"""TEST INFRASTRUCTURE: Python face of the C partition oracle (plan_oracle.c).

`build()` compiles the C file with gcc; `plan()` calls it.  The arithmetic lives
in the C file, which states which passages of the paper it follows (section
"Micro-batch Construction", Eq1, Eq2, paragraph "Limit memory consumption").
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "plan_oracle.c")
_LIB = os.path.join(_HERE, "libplan_oracle.so")

COST_POLY_GPT = 0
COST_POLY_T5 = 1
COST_TABLE = 2


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_plan.restype = ctypes.c_int
    return _lib


class OraclePlanError(Exception):
    def __init__(self, code):
        super().__init__("oracle_plan failed with code %d" % code)
        self.code = code


def plan(lengths, cap, num_stages, lengths_tgt=None, kind=COST_POLY_GPT, fixed=0, lin=2048, table=None):
    """Return dict(perm, cuts, objective, t_max); cuts has n_mb+1 entries over sorted positions."""
    lib = _load()
    ln = np.ascontiguousarray(lengths, dtype=np.int32)
    n = int(ln.shape[0])
    lt = None if lengths_tgt is None else np.ascontiguousarray(lengths_tgt, dtype=np.int32)
    tb = tl = 0
    tab = None
    if table is not None:
        tab = np.ascontiguousarray(table, dtype=np.int64)
        tb, tl = tab.shape
    perm = np.zeros(max(n, 1), dtype=np.int32)
    cuts = np.zeros(max(n, 1) + 1, dtype=np.int32)
    n_mb = ctypes.c_int32(0)
    obj = ctypes.c_int64(0)
    tmax = ctypes.c_int64(0)
    p = lambda a: None if a is None else a.ctypes.data_as(ctypes.c_void_p)
    rc = lib.oracle_plan(p(ln), p(lt), ctypes.c_int32(n), ctypes.c_int32(kind),
                         ctypes.c_int64(fixed), ctypes.c_int64(lin), p(tab),
                         ctypes.c_int32(tb), ctypes.c_int32(tl), ctypes.c_int64(cap),
                         ctypes.c_int32(num_stages), p(perm), p(cuts),
                         ctypes.byref(n_mb), ctypes.byref(obj), ctypes.byref(tmax))
    if rc != 0:
        raise OraclePlanError(rc)
    m = n_mb.value
    return {"perm": perm[:n].copy(), "cuts": cuts[:m + 1].copy(), "objective": obj.value, "t_max": tmax.value}
