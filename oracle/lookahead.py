"""ctypes front end of the C oracle of the load-look-ahead map in KV-token units
(``lookahead.c``, paper Sec. 3.4.1), plus the paper's update rule written out on fractions.

TEST INFRASTRUCTURE ONLY; see the header of ``lookahead.c``.  The C file is compiled with the
host compiler on first use if its shared object is missing or stale."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lookahead.c")
_LIB = os.path.join(_HERE, "libpso_lookahead.so")
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
        lib.pso_lookahead_update.restype = ctypes.c_int
        lib.pso_lookahead_update.argtypes = [p32, p32, p32, p32, p32, p32, ctypes.c_int64, ctypes.c_int32,
                                             ctypes.c_int32, p32, p64, p64]
        _lib = lib
    return _lib


def lookahead_update(instance_id, start_iter, prompt_tokens, i_begin, i_end, sign, n_inst: int, map_len: int,
                     kv_tokens: Optional[np.ndarray] = None,
                     overflow: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Accumulate the records into (copies of) ``kv_tokens`` [n_inst, map_len] int32 and ``overflow``
    [n_inst] int64.  Returns (kv_tokens, overflow, status, first_bad_index)."""
    lib = _load()
    c = lambda x: np.ascontiguousarray(x, dtype=np.int32)
    cols = [c(a) for a in (instance_id, start_iter, prompt_tokens, i_begin, i_end, sign)]
    n = cols[0].shape[0]
    assert all(a.shape == (n,) for a in cols)
    kv = (np.zeros((n_inst, map_len), np.int32) if kv_tokens is None
          else np.array(kv_tokens, np.int32).reshape(n_inst, map_len))
    ov = np.zeros(n_inst, np.int64) if overflow is None else np.array(overflow, np.int64)
    p32, p64 = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    bad = ctypes.c_int64(-1)
    st = lib.pso_lookahead_update(*[a.ctypes.data_as(p32) for a in cols], n, n_inst, map_len,
                                  kv.ctypes.data_as(p32), ov.ctypes.data_as(p64), ctypes.byref(bad))
    if st < 0:
        raise MemoryError("pso_lookahead_update")
    return kv, ov, st, int(bad.value)


def fraction(kv_tokens: np.ndarray, capacity) -> np.ndarray:
    """U = N / M per instance (Sec. 3.4.1: the map records the fraction of the token capacity M)."""
    cap = np.asarray(capacity, np.float64).reshape(-1, 1)
    return np.asarray(kv_tokens, np.float64) / cap


def paper_rule_on_fractions(U: np.ndarray, M: float, s: int, P: int, D: int, sign: int = 1,
                            i_begin: int = 0) -> np.ndarray:
    """The section's update exactly as printed, on the fractions of one instance:
    U'_i = (U_i * M +- (P + i)) / M for i in [i_begin, D), slot s + i.  Returns a new array."""
    U = np.array(U, np.float64)
    for i in range(i_begin, D):
        if s + i < U.shape[0]:
            U[s + i] = (U[s + i] * M + sign * (P + i)) / M
    return U
