"""One call of the hot path captured into a HIP graph and replayed on changing inputs (how the latency
configuration is served: micro-batches of 8 on the 6-layer encoder, ps_predict_load then ps_anticipate_static):
every replay must give the bits of the same call issued launch by launch.  The library's calls enqueue kernels
only (no allocation, no memset, no synchronisation), which is what makes them capturable; sizes that vary from
batch to batch live in device memory (offsets), the capture fixes only the capacity."""
import os

import numpy as np
import pytest
import torch

from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_graph_replays_match_eager_calls(tmp_models):
    cfg = wl.MODELS["latency"]
    path = os.path.join(tmp_models, "latency.bin")
    if not os.path.exists(path):
        wl.write_model(path, cfg, wl.make_weights(cfg, seed=0))
    model = ps.ps_model_load(path, 0)
    micro, cap = 8, 8 * 512
    n_inst, horizon = 4, 64
    rate = torch.tensor([30, 45, 60, 38], dtype=torch.int32, device=DEV)
    stage_ids = torch.zeros(cap, dtype=torch.int32, device=DEV)
    stage_offs = torch.zeros(micro + 1, dtype=torch.int32, device=DEV)
    stage_inst = torch.zeros(micro, dtype=torch.int32, device=DEV)
    stage_arr = torch.zeros(micro, dtype=torch.int32, device=DEV)
    pred_f = torch.empty(micro, dtype=torch.float32, device=DEV)
    pred_t = torch.empty(micro, dtype=torch.int32, device=DEV)
    load = torch.zeros(n_inst * horizon, dtype=torch.int32, device=DEV)
    ovf = torch.zeros(n_inst, dtype=torch.int64, device=DEV)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, cap, micro), DEV)
    status = ps.new_status(DEV)

    def call():
        ps.ps_predict_load(model, stage_ids, stage_offs, None, pred_f, pred_t, ws, status)
        ps.ps_anticipate_static(pred_t, stage_inst, stage_arr, rate, n_inst, horizon, load, ovf, status)

    def stage(batch, inst, arr):
        stage_ids.zero_()
        stage_ids[: batch.token_ids.size] = torch.from_numpy(batch.token_ids).to(DEV)
        stage_offs.copy_(torch.from_numpy(batch.offsets).to(DEV))
        stage_inst.copy_(torch.from_numpy(inst).to(DEV))
        stage_arr.copy_(torch.from_numpy(arr).to(DEV))

    rng = np.random.default_rng(3)
    batches = [wl.make_prompts("latency", seed=s) for s in (0, 1, 2, 3)]
    extra = [(rng.integers(0, n_inst, micro, dtype=np.int32), rng.integers(0, horizon, micro, dtype=np.int32)) for _ in batches]
    # eager results first (the map accumulates, so it is zeroed per batch)
    want = []
    for b, (inst, arr) in zip(batches, extra):
        stage(b, inst, arr)
        load.zero_(); ovf.zero_()
        call()
        torch.cuda.synchronize()
        want.append((pred_f.cpu().numpy().copy(), pred_t.cpu().numpy().copy(), load.cpu().numpy().copy(), ovf.cpu().numpy().copy()))
    assert ps.ps_status_read(status)[0] == 0
    assert len({w[0].tobytes() for w in want}) == len(want)               # the batches differ
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        call()                                                            # nothing left to set up inside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
    # replays in a mixed order, with eager work and synchronisation between them
    for it, i in enumerate([2, 0, 3, 1, 1, 2, 0]):
        print(f"graph replay {it}: micro-batch {i}", flush=True)
        inst, arr = extra[i]
        stage(batches[i], inst, arr)
        load.zero_(); ovf.zero_()
        pred_f.fill_(-1.0); pred_t.fill_(-7)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        got = (pred_f.cpu().numpy(), pred_t.cpu().numpy(), load.cpu().numpy(), ovf.cpu().numpy())
        for g, w in zip(got, want[i]):
            assert np.array_equal(g, w), f"replay {it} of micro-batch {i}"
        (torch.ones(1000, device=DEV) * 2).sum().item()                   # unrelated eager work between replays
    assert ps.ps_status_read(status)[0] == 0
