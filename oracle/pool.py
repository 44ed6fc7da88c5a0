"""Runs the fp64 predictor oracle over many requests on several host cores.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only tests and the benchmark's CPU-baseline leg use it.

A request's prediction depends on nothing but its own tokens, so the requests are dealt to worker
processes (this file run as a program), each with its own copy of the model read from the model
file.  The workers import only the oracle and numpy and run single-threaded; the process that
starts them may hold a GPU context, they never touch it.

    python -m oracle.pool <model file> <requests .npz> <output .npy>
"""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from typing import Sequence

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def workers_available(limit: int = 16) -> int:
    """Host cores this process may use, at most `limit` (a GPU machine gives one GPU's share of its cores)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(limit, n))


def predict_requests(model_path: str, requests: Sequence[np.ndarray], workers: int = 0,
                     timeout_s: float = 900.0) -> np.ndarray:
    """pred_f (fp64) of every request (an array of its text token ids)."""
    n = len(requests)
    workers = max(1, min(workers or workers_available(), n))
    # longest first, each to the worker with the least work so far (cost ~ tokens, plus a share per request
    # for streaming the weights once)
    cost = np.array([len(r) + 64 for r in requests], np.int64)
    load = np.zeros(workers, np.int64)
    share = [[] for _ in range(workers)]
    for i in np.argsort(-cost, kind="stable"):
        w = int(np.argmin(load))
        share[w].append(int(i))
        load[w] += cost[i]
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    out = np.empty(n, np.float64)
    with tempfile.TemporaryDirectory() as tmp:
        procs = []
        for w in range(workers):
            src, dst = os.path.join(tmp, f"in{w}.npz"), os.path.join(tmp, f"out{w}.npy")
            lens = np.array([len(requests[i]) for i in share[w]], np.int64)
            ids = np.concatenate([np.asarray(requests[i], np.int64) for i in share[w]]) if share[w] else np.zeros(0, np.int64)
            np.savez(src, lengths=lens, ids=ids)
            procs.append((subprocess.Popen([sys.executable, "-m", "oracle.pool", model_path, src, dst],
                                           cwd=ROOT, env=env), dst))
        try:
            for w, (p, dst) in enumerate(procs):
                if p.wait(timeout=timeout_s) != 0:
                    raise RuntimeError(f"oracle worker {w} failed with exit code {p.returncode}")
                out[share[w]] = np.load(dst)
        finally:
            for p, _ in procs:
                if p.poll() is None:
                    p.kill()
    return out


def _worker(model_path: str, src: str, dst: str) -> None:
    from oracle import predictor as op
    model = op.load_model(model_path)
    data = np.load(src)
    ends = np.cumsum(data["lengths"])
    vals = np.empty(len(ends), np.float64)
    for j, end in enumerate(ends):
        ids = data["ids"][end - data["lengths"][j]: end]
        vals[j] = op.regression_head(model, op.encode_request(model, ids)[0])
    np.save(dst, vals)


if __name__ == "__main__":
    _worker(*sys.argv[1:4])
