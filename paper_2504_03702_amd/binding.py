"""Thin ctypes binding over the C-ABI library (``include/preserve.h``), same names as the C calls.

Argument marshalling only: tensors supply device pointers, ``torch.cuda.current_stream()`` the
stream; every step of the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing or there is no GPU the calls raise."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpreserve.so")

PS_OK = 0
PS_ERRORS = {-1: "PS_EINVAL", -2: "PS_EIO", -3: "PS_EFORMAT", -4: "PS_ENOMEM", -5: "PS_EWORKSPACE",
             -6: "PS_EUNSUPPORTED", -7: "PS_EHIP"}
PS_ST_BAD_TOKEN, PS_ST_BAD_LENGTH, PS_ST_NAN, PS_ST_BAD_RECORD, PS_ST_RANGE = 0x01, 0x02, 0x04, 0x10, 0x20

EXPORTS = ["ps_model_load", "ps_model_free", "ps_model_get_info", "ps_workspace_bytes", "ps_predict_load",
           "ps_anticipate_workspace_bytes", "ps_anticipate", "ps_anticipate_static", "ps_status_read", "ps_strerror",
           "ps_profile_enable", "ps_profile_read", "ps_profile_clock", "ps_profile_stream_read",
           "ps_lookahead_workspace_bytes", "ps_lookahead_update", "ps_scaler_scan", "ps_route", "ps_forecast"]
PS_FAMILIES = ["embed", "gemm", "attention", "layernorm", "head", "refine"]


class PsError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {PS_ERRORS.get(code, code)}")
        self.code = code


class ps_model_info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("layers", "hidden", "heads", "ffn", "vocab", "max_pos",
                                              "n_soft", "head_hidden", "dtype", "d_max")]


class ps_status(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_int32), ("reserved", ctypes.c_int32), ("first_bad", ctypes.c_int64)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load ``libpreserve.so`` (built in-tree by ``build.py``) and declare its entry points."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run paper_2504_03702_amd/build.py")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.ps_model_load.restype = ctypes.c_int
    lib.ps_model_load.argtypes = [ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(vp)]
    lib.ps_model_free.restype = None
    lib.ps_model_free.argtypes = [vp]
    lib.ps_model_get_info.restype = ctypes.c_int
    lib.ps_model_get_info.argtypes = [vp, ctypes.POINTER(ps_model_info)]
    lib.ps_workspace_bytes.restype = sz
    lib.ps_workspace_bytes.argtypes = [vp, i64, i32]
    lib.ps_predict_load.restype = ctypes.c_int
    lib.ps_predict_load.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp, sz, vp, vp]
    lib.ps_anticipate_workspace_bytes.restype = sz
    lib.ps_anticipate_workspace_bytes.argtypes = [i64, i32, i32]
    lib.ps_anticipate.restype = ctypes.c_int
    lib.ps_anticipate.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, vp, vp, sz, vp, vp]
    lib.ps_anticipate_static.restype = ctypes.c_int
    lib.ps_anticipate_static.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp]
    lib.ps_lookahead_workspace_bytes.restype = sz
    lib.ps_lookahead_workspace_bytes.argtypes = [i64, i32, i32]
    lib.ps_lookahead_update.restype = ctypes.c_int
    lib.ps_lookahead_update.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.ps_scaler_scan.restype = ctypes.c_int
    lib.ps_scaler_scan.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.ps_route.restype = ctypes.c_int
    lib.ps_route.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.ps_forecast.restype = ctypes.c_int
    lib.ps_forecast.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, vp]
    lib.ps_status_read.restype = ctypes.c_int
    lib.ps_status_read.argtypes = [vp, vp, ctypes.POINTER(ps_status)]
    lib.ps_profile_enable.restype = ctypes.c_int
    lib.ps_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.ps_profile_read.restype = ctypes.c_int
    lib.ps_profile_read.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.ps_profile_clock.restype = ctypes.c_int
    lib.ps_profile_clock.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.ps_profile_stream_read.restype = ctypes.c_int
    lib.ps_profile_stream_read.argtypes = [vp, ctypes.c_int64, vp, vp]
    lib.ps_strerror.restype = ctypes.c_char_p
    lib.ps_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(code: int, where: str) -> None:
    if code != PS_OK:
        raise PsError(code, where)


class Model:
    """Owner of a ``ps_model*``."""

    def __init__(self, handle: int, device: int):
        self.handle, self.device = handle, device
        info = ps_model_info()
        _check(load_library().ps_model_get_info(handle, ctypes.byref(info)), "ps_model_get_info")
        self.info = info

    def close(self) -> None:
        if self.handle:
            load_library().ps_model_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ps_model_load(path: str, device: int = 0) -> Model:
    if not torch.cuda.is_available():
        raise RuntimeError("ps_model_load needs a GPU")
    out = ctypes.c_void_p()
    _check(load_library().ps_model_load(os.fsencode(path), device, ctypes.byref(out)), "ps_model_load")
    return Model(out.value, device)


def ps_profile_enable(model: Model, on: bool) -> None:
    _check(load_library().ps_profile_enable(model.handle, int(on)), "ps_profile_enable")


def ps_profile_read(model: Model) -> dict:
    """{family: (milliseconds, launches)} since the last read; waits for the current stream."""
    n = len(PS_FAMILIES)
    ms, cnt = (ctypes.c_double * n)(), (ctypes.c_int64 * n)()
    _check(load_library().ps_profile_read(model.handle, _stream(), ms, cnt), "ps_profile_read")
    return {f: (float(ms[i]), int(cnt[i])) for i, f in enumerate(PS_FAMILIES)}


def ps_profile_clock(model: Model) -> float:
    """Core clock (GHz) sustained during the last large GEMM launched while profiling was on; 0 if none."""
    ghz = ctypes.c_double(0.0)
    _check(load_library().ps_profile_clock(model.handle, _stream(), ctypes.byref(ghz)), "ps_profile_clock")
    return float(ghz.value)


def ps_profile_stream_read(data: torch.Tensor, sink: torch.Tensor, nbytes: Optional[int] = None) -> None:
    """Enqueue the read-only yardstick kernel over the first nbytes of `data` (all of it by default); the XOR
    of its 64-bit words is accumulated into sink[0] (int64 / uint64 device tensor)."""
    n = data.numel() * data.element_size() if nbytes is None else int(nbytes)
    _check(load_library().ps_profile_stream_read(data.data_ptr(), n, sink.data_ptr(), _stream()),
           "ps_profile_stream_read")


def ps_workspace_bytes(model: Model, max_tokens: int, max_req: int) -> int:
    return int(load_library().ps_workspace_bytes(model.handle, max_tokens, max_req))


def new_status(device="cuda") -> torch.Tensor:
    """A zeroed device ps_status block (two int64 words)."""
    return torch.zeros(2, dtype=torch.int64, device=device)


def ps_status_read(status: torch.Tensor) -> Tuple[int, int]:
    """(flags, first_bad) after waiting for the current stream."""
    out = ps_status()
    _check(load_library().ps_status_read(_ptr(status, torch.int64, "status"), _stream(), ctypes.byref(out)),
           "ps_status_read")
    return int(out.flags), int(out.first_bad)


def ps_predict_load(model: Model, token_ids: torch.Tensor, offsets: torch.Tensor,
                    lengths: Optional[torch.Tensor], pred_f: torch.Tensor, pred_tokens: torch.Tensor,
                    workspace: torch.Tensor, status: Optional[torch.Tensor] = None) -> None:
    n_req = offsets.numel() - 1
    _check(load_library().ps_predict_load(
        model.handle, _ptr(token_ids, torch.int32, "token_ids"), _ptr(offsets, torch.int32, "offsets"),
        _ptr(lengths, torch.int32, "lengths"), n_req, token_ids.numel(),
        _ptr(pred_f, torch.float32, "pred_f"), _ptr(pred_tokens, torch.int32, "pred_tokens"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _ptr(status, torch.int64, "status"), _stream()), "ps_predict_load")


def ps_anticipate_workspace_bytes(n_req: int, n_inst: int, horizon: int) -> int:
    return int(load_library().ps_anticipate_workspace_bytes(n_req, n_inst, horizon))


def ps_anticipate(pred_tokens: torch.Tensor, instance_id: torch.Tensor, arrival_bucket: torch.Tensor,
                  rate: Optional[torch.Tensor], n_inst: int, horizon: int, load: torch.Tensor,
                  overflow: Optional[torch.Tensor], workspace: torch.Tensor,
                  status: Optional[torch.Tensor] = None) -> None:
    if load.numel() != n_inst * horizon or (overflow is not None and overflow.numel() != n_inst) or \
            (rate is not None and rate.numel() != n_inst) or \
            instance_id.numel() != pred_tokens.numel() or arrival_bucket.numel() != pred_tokens.numel():
        raise ValueError("ps_anticipate: array sizes do not match n_req / n_inst / horizon")
    _check(load_library().ps_anticipate(
        _ptr(pred_tokens, torch.int32, "pred_tokens"), _ptr(instance_id, torch.int32, "instance_id"),
        _ptr(arrival_bucket, torch.int32, "arrival_bucket"), _ptr(rate, torch.int32, "rate"),
        pred_tokens.numel(), n_inst, horizon, _ptr(load, torch.int32, "load"),
        _ptr(overflow, torch.int64, "overflow"), _ptr(workspace, torch.uint8, "workspace"),
        workspace.numel(), _ptr(status, torch.int64, "status"), _stream()), "ps_anticipate")


PS_ANTICIPATE_STATIC_BYTES = 8 << 20


def ps_anticipate_static(pred_tokens: torch.Tensor, instance_id: torch.Tensor, arrival_bucket: torch.Tensor,
                         rate: Optional[torch.Tensor], n_inst: int, horizon: int, load: torch.Tensor,
                         overflow: Optional[torch.Tensor], status: Optional[torch.Tensor] = None) -> None:
    """ps_anticipate without a workspace argument: the library's own fixed device array holds the partial curves."""
    if load.numel() != n_inst * horizon or (overflow is not None and overflow.numel() != n_inst) or \
            (rate is not None and rate.numel() != n_inst) or \
            instance_id.numel() != pred_tokens.numel() or arrival_bucket.numel() != pred_tokens.numel():
        raise ValueError("ps_anticipate_static: array sizes do not match n_req / n_inst / horizon")
    _check(load_library().ps_anticipate_static(
        _ptr(pred_tokens, torch.int32, "pred_tokens"), _ptr(instance_id, torch.int32, "instance_id"),
        _ptr(arrival_bucket, torch.int32, "arrival_bucket"), _ptr(rate, torch.int32, "rate"),
        pred_tokens.numel(), n_inst, horizon, _ptr(load, torch.int32, "load"),
        _ptr(overflow, torch.int64, "overflow"), _ptr(status, torch.int64, "status"), _stream()),
        "ps_anticipate_static")


def ps_lookahead_workspace_bytes(n_rec: int, n_inst: int, map_len: int) -> int:
    return int(load_library().ps_lookahead_workspace_bytes(n_rec, n_inst, map_len))


def ps_lookahead_update(instance_id: torch.Tensor, start_iter: torch.Tensor, prompt_tokens: torch.Tensor,
                        i_begin: torch.Tensor, i_end: torch.Tensor, sign: torch.Tensor, n_inst: int, map_len: int,
                        kv_tokens: torch.Tensor, overflow: Optional[torch.Tensor], workspace: torch.Tensor,
                        capacity: Optional[torch.Tensor] = None, fraction: Optional[torch.Tensor] = None,
                        status: Optional[torch.Tensor] = None) -> None:
    cols = (instance_id, start_iter, prompt_tokens, i_begin, i_end, sign)
    n = instance_id.numel()
    if any(c.numel() != n for c in cols) or kv_tokens.numel() != n_inst * map_len or \
            (overflow is not None and overflow.numel() != n_inst) or \
            (capacity is not None and capacity.numel() != n_inst) or \
            (fraction is not None and fraction.numel() != n_inst * map_len):
        raise ValueError("ps_lookahead_update: array sizes do not match n_rec / n_inst / map_len")
    names = ("instance_id", "start_iter", "prompt_tokens", "i_begin", "i_end", "sign")
    _check(load_library().ps_lookahead_update(
        *[_ptr(c, torch.int32, nm) for c, nm in zip(cols, names)], n, n_inst, map_len,
        _ptr(kv_tokens, torch.int32, "kv_tokens"), _ptr(overflow, torch.int64, "overflow"),
        _ptr(capacity, torch.int32, "capacity"), _ptr(fraction, torch.float32, "fraction"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _ptr(status, torch.int64, "status"),
        _stream()), "ps_lookahead_update")


def ps_scaler_scan(kv_tokens: torch.Tensor, capacity: torch.Tensor, n_inst: int, map_len: int, window: int,
                   over_count: torch.Tensor, peak_tokens: torch.Tensor, overloaded: torch.Tensor,
                   summary: torch.Tensor, scale_down: torch.Tensor, over_pct: int = 95, share_pct: int = 10,
                   idle_pct: int = 30) -> None:
    if kv_tokens.numel() != n_inst * map_len or capacity.numel() != n_inst or summary.numel() != 2 or \
            scale_down.numel() != 1 or any(t.numel() != n_inst for t in (over_count, peak_tokens, overloaded)):
        raise ValueError("ps_scaler_scan: array sizes do not match n_inst / map_len")
    _check(load_library().ps_scaler_scan(
        _ptr(kv_tokens, torch.int32, "kv_tokens"), _ptr(capacity, torch.int32, "capacity"), n_inst, map_len, window,
        over_pct, share_pct, idle_pct, _ptr(over_count, torch.int32, "over_count"),
        _ptr(peak_tokens, torch.int32, "peak_tokens"), _ptr(overloaded, torch.int32, "overloaded"),
        _ptr(summary, torch.int32, "summary"), _ptr(scale_down, torch.float64, "scale_down"), _stream()),
        "ps_scaler_scan")


def ps_route(prompt_tokens: torch.Tensor, pred_tokens: torch.Tensor, n_inst: int, window: int,
             window_tokens: Optional[torch.Tensor], capacity: torch.Tensor, queued_p: torch.Tensor,
             current_d: torch.Tensor, assigned: torch.Tensor, score100: torch.Tensor, t_mem_pct: int = 80,
             beta: int = 1, status: Optional[torch.Tensor] = None) -> None:
    n = prompt_tokens.numel()
    if pred_tokens.numel() != n or assigned.numel() != n or score100.numel() != n or capacity.numel() != n_inst or \
            queued_p.numel() != n_inst or current_d.numel() != n_inst or \
            (window_tokens is not None and window_tokens.numel() != n_inst * window):
        raise ValueError("ps_route: array sizes do not match n_req / n_inst / window")
    _check(load_library().ps_route(
        _ptr(prompt_tokens, torch.int32, "prompt_tokens"), _ptr(pred_tokens, torch.int32, "pred_tokens"), n, n_inst,
        window, _ptr(window_tokens, torch.int32, "window_tokens"), _ptr(capacity, torch.int32, "capacity"),
        _ptr(queued_p, torch.int64, "queued_p"), _ptr(current_d, torch.int64, "current_d"), t_mem_pct, beta,
        _ptr(assigned, torch.int32, "assigned"), _ptr(score100, torch.int64, "score100"),
        _ptr(status, torch.int64, "status"), _stream()), "ps_route")


def ps_forecast(weights: torch.Tensor, hidden: int, hist_p: torch.Tensor, hist_d: torch.Tensor, n_services: int,
                k: int, mu: torch.Tensor, out: torch.Tensor) -> None:
    if weights.numel() != n_services * 2 * (5 * hidden * hidden + 10 * hidden + 1) or hist_p.numel() != n_services * k or \
            hist_d.numel() != n_services * k or mu.numel() != 3 * n_services or out.numel() != 5 * n_services:
        raise ValueError("ps_forecast: array sizes do not match n_services / hidden / k")
    _check(load_library().ps_forecast(
        _ptr(weights, torch.float32, "weights"), hidden, _ptr(hist_p, torch.float32, "hist_p"),
        _ptr(hist_d, torch.float32, "hist_d"), n_services, k, _ptr(mu, torch.float32, "mu"),
        _ptr(out, torch.float32, "out"), _stream()), "ps_forecast")


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Uninitialised device scratch; torch's allocator hands out 512-byte aligned blocks."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
