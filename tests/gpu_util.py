"""Helpers shared by the GPU parity tests: run the library on numpy inputs, error metric."""
import numpy as np
import torch

from paper_2504_03702_amd import binding as ps

# |gpu - oracle| <= tol * max(|oracle|, rms(oracle)): relative error, with the batch's RMS as the
# floor because a pure relative error is undefined for predictions near zero.
TOL_FP32 = 1e-4
TOL_BF16 = 1e-2


def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref ** 2)))
    return np.abs(got - ref) / scale


def run_predict(model, batch, dev="cuda:0", status=None):
    n = batch.n_req
    ids = torch.from_numpy(np.ascontiguousarray(batch.token_ids, np.int32)).to(dev)
    offs = torch.from_numpy(np.ascontiguousarray(batch.offsets, np.int32)).to(dev)
    lens = None if batch.lengths is None else torch.from_numpy(np.ascontiguousarray(batch.lengths, np.int32)).to(dev)
    pred_f = torch.full((n,), 12345.0, dtype=torch.float32, device=dev)
    pred_t = torch.full((n,), -7, dtype=torch.int32, device=dev)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, ids.numel(), n), dev)
    st = ps.new_status(dev) if status is None else status
    ps.ps_predict_load(model, ids, offs, lens, pred_f, pred_t, ws, st)
    flags, bad = ps.ps_status_read(st)
    return pred_f.cpu().numpy(), pred_t.cpu().numpy(), flags, bad


def run_anticipate(inp, load=None, overflow=None, dev="cuda:0"):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    n = int(inp.pred_tokens.shape[0])
    load_t = torch.zeros(inp.n_inst * inp.horizon, dtype=torch.int32, device=dev) if load is None \
        else torch.from_numpy(np.ascontiguousarray(load, np.int32).reshape(-1)).to(dev)
    ovf_t = torch.zeros(inp.n_inst, dtype=torch.int64, device=dev) if overflow is None \
        else torch.from_numpy(np.ascontiguousarray(overflow, np.int64)).to(dev)
    rate = None if inp.rate is None else t(inp.rate)
    ws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(n, inp.n_inst, inp.horizon), dev)
    st = ps.new_status(dev)
    ps.ps_anticipate(t(inp.pred_tokens), t(inp.instance_id), t(inp.arrival_bucket), rate, inp.n_inst,
                     inp.horizon, load_t, ovf_t, ws, st)
    flags, bad = ps.ps_status_read(st)
    return load_t.cpu().numpy().reshape(inp.n_inst, inp.horizon), ovf_t.cpu().numpy(), flags, bad


def run_lookahead(cols, n_inst, map_len, kv=None, overflow=None, capacity=None, want_fraction=False,
                  with_overflow=True, dev="cuda:0"):
    """ps_lookahead_update on numpy columns (instance, start, prompt, i_begin, i_end, sign).
    Returns (kv_tokens, overflow, fraction or None, flags, first_bad)."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    kv_t = torch.zeros(n_inst * map_len, dtype=torch.int32, device=dev) if kv is None \
        else torch.from_numpy(np.ascontiguousarray(kv, np.int32).reshape(-1)).to(dev)
    ovf_t = None
    if with_overflow:
        ovf_t = torch.zeros(n_inst, dtype=torch.int64, device=dev) if overflow is None \
            else torch.from_numpy(np.ascontiguousarray(overflow, np.int64)).to(dev)
    cap_t = None if capacity is None else t(capacity)
    frac_t = torch.full((n_inst * map_len,), -1.0, dtype=torch.float32, device=dev) if want_fraction else None
    ws = ps.alloc_workspace(ps.ps_lookahead_workspace_bytes(len(cols[0]), n_inst, map_len), dev)
    ws.fill_(0xA5)                               # the library must not rely on a clean workspace
    st = ps.new_status(dev)
    ps.ps_lookahead_update(*[t(c) for c in cols], n_inst, map_len, kv_t, ovf_t, ws, cap_t, frac_t, st)
    flags, bad = ps.ps_status_read(st)
    return (kv_t.cpu().numpy().reshape(n_inst, map_len), None if ovf_t is None else ovf_t.cpu().numpy(),
            None if frac_t is None else frac_t.cpu().numpy().reshape(n_inst, map_len), flags, bad)
