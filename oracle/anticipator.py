"""ctypes front end of the C anticipator oracle (``anticipator.c``).

TEST INFRASTRUCTURE ONLY; see the header of ``anticipator.c``.  The C file is compiled
with the host compiler on first use if its shared object is missing or stale."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "anticipator.c")
_LIB = os.path.join(_HERE, "libpso_anticipator.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-shared", "-fPIC", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p32, p64 = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        lib.pso_anticipate.restype = ctypes.c_int
        lib.pso_anticipate.argtypes = [p32, p32, p32, p32, ctypes.c_int64, ctypes.c_int32,
                                       ctypes.c_int32, p32, p64, p64]
        _lib = lib
    return _lib


def anticipate(pred_tokens, instance_id, arrival_bucket, rate: Optional[np.ndarray],
               n_inst: int, horizon: int, load: Optional[np.ndarray] = None,
               overflow: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Accumulate into (copies of) ``load`` [n_inst, horizon] int32 and ``overflow`` [n_inst]
    int64.  Returns (load, overflow, status, first_bad_index)."""
    lib = _load()
    c = lambda x: np.ascontiguousarray(x, dtype=np.int32)
    pred, inst, arr = c(pred_tokens), c(instance_id), c(arrival_bucket)
    n = pred.shape[0]
    assert inst.shape[0] == n and arr.shape[0] == n
    load = np.zeros((n_inst, horizon), np.int32) if load is None else np.array(load, np.int32).reshape(n_inst, horizon)
    overflow = np.zeros(n_inst, np.int64) if overflow is None else np.array(overflow, np.int64)
    p32, p64 = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    rp = None
    if rate is not None:
        rate = c(rate)
        assert rate.shape[0] == n_inst
        rp = rate.ctypes.data_as(p32)
    bad = ctypes.c_int64(-1)
    st = lib.pso_anticipate(pred.ctypes.data_as(p32), inst.ctypes.data_as(p32), arr.ctypes.data_as(p32),
                            rp, n, n_inst, horizon, load.ctypes.data_as(p32),
                            overflow.ctypes.data_as(p64), ctypes.byref(bad))
    if st < 0:
        raise MemoryError("pso_anticipate")
    return load, overflow, st, int(bad.value)
