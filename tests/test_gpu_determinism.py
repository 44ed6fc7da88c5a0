"""Run-twice bit-compare: the same call on the same inputs gives the same bits, whatever the workgroups' timing
(fixed orders of floating-point additions in the predictor; integer sums in the map kernels, where a race
would show as a changed histogram)."""
import os

import numpy as np
import pytest

from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
from tests.gpu_util import run_anticipate, run_lookahead, run_predict

pytestmark = pytest.mark.gpu


def test_predictor_twice(tmp_models):
    cfg = wl.MODELS["bert_base"]
    path = os.path.join(tmp_models, "bert_base.bin")
    if not os.path.exists(path):
        wl.write_model(path, cfg, wl.make_weights(cfg, seed=0))
    model = ps.ps_model_load(path, 0)
    for kind, n in (("bert_base_varlen", 600), ("latency", 8)):
        print(f"determinism predictor {kind}", flush=True)
        batch = wl.make_prompts(kind, seed=5, n_req=n)
        a = run_predict(model, batch)
        b = run_predict(model, batch)
        assert a[2] == 0 and np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_map_kernels_twice():
    for kind, n in (("stream", 2_000_001), ("stream_by_arrival", 2_000_001), ("production", 4096)):
        print(f"determinism anticipator {kind}", flush=True)
        inp = wl.make_anticipator_inputs(kind, seed=8, n=n)
        a, b = run_anticipate(inp), run_anticipate(inp)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2] == 0
    x = wl.make_lookahead_inputs("production", seed=8, n=300_000)
    a = run_lookahead(x.columns(), x.n_inst, x.map_len, capacity=x.capacity, want_fraction=True)
    b = run_lookahead(x.columns(), x.n_inst, x.map_len, capacity=x.capacity, want_fraction=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
