#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: requests predicted per second.

A step is one pass of the whole path over one batch of synthetic prompts already resident in
HBM: ps_predict_load (gather, encoder, head) followed on the same stream by ps_anticipate on the
predictions.  Prints one JSON line with the throughput, the roofline of the dominant kernel (the
bf16 MFMA GEMM; duration from HIP events the library records around every launch in the timed
region), the anticipator's HBM rate on a long record stream, and the CPU oracle timed on a bounded
sample of the same workload on this machine's host cores."""
from __future__ import annotations

import argparse
import json
import os
import sys
import tempfile
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak

# Bytes that left the L2 caches per large-GEMM launch (average over the 61 launches of a production
# step), from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; profiles/production_gemm_traffic.txt)
# scaled by what the same counters read for a 1 GiB elementwise copy (x2.0 and x1.0).  Valid only for
# the kernel source it was measured on: reported as null once that file has changed.
GEMM_TRAFFIC = {"source_sha256_16": "2235e98ece3ba0d0", "workload": "production",
                "fetch_bytes": 23.077e9, "write_bytes": 10.115e9}


def measured_gemm_traffic(workload: str):
    import hashlib
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2504_03702_amd", "csrc", "gemm_bf16.hip")
    try:
        with open(src, "rb") as f:
            digest = hashlib.sha256(f.read()).hexdigest()[:16]
    except OSError:
        return None
    if digest != GEMM_TRAFFIC["source_sha256_16"] or workload != GEMM_TRAFFIC["workload"]:
        return None
    return GEMM_TRAFFIC["fetch_bytes"] + GEMM_TRAFFIC["write_bytes"]

# workload name -> (encoder shape, prompt recipe, anticipator recipe, description)
WORKLOADS = {
    "tiny": ("tiny", "tiny", "tiny", "2-layer H128 fp32 encoder, 16 prompts of 8-64 tokens; anticipator 4x64"),
    "bert_base_padded": ("bert_base", "bert_base_padded", "small",
                         "BERT-base-shaped bf16 encoder, 64 prompts padded to the batch maximum; anticipator 4x64"),
    "bert_base_varlen": ("bert_base", "bert_base_varlen", "medium",
                         "BERT-base-shaped bf16 encoder, 1024 packed prompts (lognormal lengths, Zipf ids); "
                         "anticipator 64x600"),
    "latency": ("latency", "latency", "small", "6-layer H768 bf16 encoder, micro-batches of 8 prompts; anticipator 4x64"),
    "production": ("production", "production", "production",
                   "16-layer H1024 A16 F4096 bf16 encoder, 4096 packed prompts (lognormal(5.5,1.2) in [4,2048]); "
                   "anticipator 256 instances x 600 buckets, rates 30-60 tok/s"),
}


def encoder_flops(cfg, lengths):
    """Flops of the work one call asks of the GEMM and attention kernels, on real tokens.  In the last
    layer only the first row of every request goes on to the head, so there the library runs the key and
    value projections alone over all rows and attention for the first rows: that is what is counted (the
    small per-request side GEMMs are left out)."""
    H, F, L = cfg.hidden, cfg.ffn, cfg.layers
    S = lengths.astype(np.float64) + cfg.n_soft
    gemm = (L - 1) * S.sum() * (8.0 * H * H + 4.0 * H * F) + S.sum() * 4.0 * H * H
    attn = (L - 1) * 4.0 * H * (S ** 2).sum() + 4.0 * H * S.sum()
    return gemm, attn


def time_cpu_oracle(model_path, batch, ant, stream=None, budget_s=8.0):
    """The fp64 oracle as it stands, on this machine's host cores, on bounded samples of the same workload:
    the predictor + anticipator on the first requests of the batch, once on one core (numpy held to one
    thread) and once over all cores this process may use (one single-threaded worker process per core, the
    requests dealt among them); and the anticipator oracle alone (C, one core) on the whole record stream the
    GPU leg times.  Samples are sized from a quick probe of this host's fp64 matmul rate."""
    from oracle import anticipator as oa
    from oracle import pool as opool
    from oracle import predictor as op
    try:
        from threadpoolctl import threadpool_limits
    except ImportError:                                   # without it numpy keeps its own thread count
        threadpool_limits = None
    model = op.load_model(model_path)
    lengths = batch.valid_lengths()
    H, F, L = model["hidden"], model["ffn"], model["layers"]
    per_req = L * (lengths * (8.0 * H * H + 4.0 * H * F) + 4.0 * H * lengths.astype(np.float64) ** 2)

    def probe():
        a = np.random.default_rng(0).standard_normal((512, 1024))
        b = np.random.default_rng(1).standard_normal((1024, 1024))
        a @ b
        t0 = time.perf_counter()
        for _ in range(3):
            a @ b
        return 3 * 2 * 512 * 1024 * 1024 / (time.perf_counter() - t0)          # flop/s

    def sample_size(flops):
        return max(1, min(int(np.searchsorted(np.cumsum(per_req), flops)) + 1, batch.n_req))

    # one core
    import contextlib
    with (threadpool_limits(limits=1) if threadpool_limits else contextlib.nullcontext()):
        rate1 = probe()
        n1 = sample_size(0.5 * rate1 * budget_s)          # the oracle's mix of operations runs at about half the probe rate
        offs = batch.offsets[: n1 + 1]
        lens = None if batch.lengths is None else batch.lengths[:n1]
        t0 = time.perf_counter()
        _, tok = op.predict_load(model, batch.token_ids, offs, lens)
        oa.anticipate(tok, ant.instance_id[:n1], ant.arrival_bucket[:n1], ant.rate, ant.n_inst, ant.horizon)
        dt1 = time.perf_counter() - t0
    threads1 = 1 if threadpool_limits else int(os.environ.get("OMP_NUM_THREADS", 0)) or (os.cpu_count() or 1)
    single = {"value": n1 / dt1, "unit": "requests/s", "cores": threads1,
              "sample": f"first {n1} requests ({int(lengths[:n1].sum())} tokens) of the batch, fp64 numpy + C, {dt1:.1f} s"}
    # all cores: worker processes, each numpy single-threaded
    cores = opool.workers_available(limit=64)
    nc = sample_size(per_req[:n1].sum() / dt1 * budget_s * cores)
    valid = batch.valid_lengths()
    reqs = [batch.token_ids[batch.offsets[r]: batch.offsets[r] + valid[r]] for r in range(nc)]
    t0 = time.perf_counter()
    pred = opool.predict_requests(model_path, reqs, workers=cores)
    tok = np.clip(np.rint(pred), 0, model["d_max"]).astype(np.int32)
    oa.anticipate(tok, ant.instance_id[:nc], ant.arrival_bucket[:nc], ant.rate, ant.n_inst, ant.horizon)
    dtc = time.perf_counter() - t0
    out = {"value": nc / dtc, "unit": "requests/s", "cores": min(cores, nc), "kind": "oracle",
           "sample": f"first {nc} requests ({int(lengths[:nc].sum())} tokens) of the batch dealt to {min(cores, nc)} "
                     f"single-threaded worker processes (model read by each included), fp64 numpy + C, {dtc:.1f} s",
           "host_cores": os.cpu_count(), "single_thread": single}
    if stream is not None:
        t0 = time.perf_counter()
        oa.anticipate(stream.pred_tokens, stream.instance_id, stream.arrival_bucket, stream.rate, stream.n_inst,
                      stream.horizon)
        dts = time.perf_counter() - t0
        n_s = int(stream.pred_tokens.shape[0])
        out["anticipator"] = {"records_per_s": n_s / dts, "GB/s": (12.0 * n_s + 8.0 * stream.n_inst * stream.horizon) / dts / 1e9,
                              "cores": 1, "sample": f"the whole {n_s}-record stream in arbitrary order, C oracle, {dts:.1f} s"}
    return out


def latency_leg(torch, ps, wl, dev, status, n_batches, warm, rate_per_s=2000.0, micro=8):
    """The latency configuration: a seeded Poisson stream of requests at `rate_per_s` served in micro-batches of
    `micro` by the 6-layer H768 encoder, ps_predict_load followed by ps_anticipate_static, replayed in real
    time: batch b becomes ready when its last request has arrived, is launched then (or as soon as the batch
    before it has finished), and its latency runs from ready to predictions and map complete on the device.
    Two ways of issuing the same kernels: one launch after the other from the host ("eager"), and the whole call
    captured once into a HIP graph on fixed staging buffers of the largest micro-batch, replayed per batch
    after one device-to-device copy of the batch's inputs ("graph")."""
    cfg = wl.MODELS["latency"].resolved()
    tmp = tempfile.mkdtemp(prefix="ps_bench_lat_")
    path = os.path.join(tmp, "latency.bin")
    wl.write_model(path, cfg, wl.make_weights(cfg, seed=0))
    model = ps.ps_model_load(path, 0)
    os.remove(path)
    os.rmdir(tmp)
    total = warm + n_batches
    n = total * micro
    big = wl.make_prompts("latency", seed=0, n_req=n)
    lengths = big.valid_lengths()
    arrivals = wl.poisson_arrival_times(0, n, rate_per_s)
    ready = arrivals[micro - 1:: micro]                                    # a batch closes with its last request
    ant = wl.make_anticipator_inputs("small", seed=0, n=n, pred_tokens=np.zeros(n, np.int32))
    bucket = np.minimum(np.floor(arrivals), ant.horizon - 1).astype(np.int32)
    cap_tokens = micro * 512                                               # token slots of the largest micro-batch
    # one staging row per batch: token ids | offsets (padded to 12) | instance | arrival bucket
    row_w = cap_tokens + 12 + 2 * micro
    rows = np.zeros((total, row_w), np.int32)
    for b in range(total):
        r0 = b * micro
        t0, t1 = big.offsets[r0], big.offsets[r0 + micro]
        rows[b, : t1 - t0] = big.token_ids[t0:t1]
        rows[b, cap_tokens: cap_tokens + micro + 1] = big.offsets[r0: r0 + micro + 1] - t0
        rows[b, cap_tokens + 12: cap_tokens + 12 + micro] = ant.instance_id[r0: r0 + micro]
        rows[b, cap_tokens + 12 + micro:] = bucket[r0: r0 + micro]
    rows_d = torch.from_numpy(rows).to(dev)
    rate_d = torch.from_numpy(ant.rate).to(dev)
    stage = torch.zeros(row_w, dtype=torch.int32, device=dev)
    s_ids, s_offs = stage[:cap_tokens], stage[cap_tokens: cap_tokens + micro + 1]
    s_inst, s_arr = stage[cap_tokens + 12: cap_tokens + 12 + micro], stage[cap_tokens + 12 + micro:]
    pred_f = torch.empty(micro, dtype=torch.float32, device=dev)
    pred_t = torch.empty(micro, dtype=torch.int32, device=dev)
    load = torch.zeros(ant.n_inst * ant.horizon, dtype=torch.int32, device=dev)
    ovf = torch.zeros(ant.n_inst, dtype=torch.int64, device=dev)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, cap_tokens, micro), dev)

    def call_on_stage():
        ps.ps_predict_load(model, s_ids, s_offs, None, pred_f, pred_t, ws, status)
        ps.ps_anticipate_static(pred_t, s_inst, s_arr, rate_d, ant.n_inst, ant.horizon, load, ovf, status)

    def eager(b):
        # the batch's own slices of the resident inputs; token slots = its real token count
        row = rows_d[b]
        n_tok = int(big.offsets[(b + 1) * micro] - big.offsets[b * micro])
        ps.ps_predict_load(model, row[:n_tok], row[cap_tokens: cap_tokens + micro + 1], None, pred_f, pred_t, ws, status)
        ps.ps_anticipate_static(pred_t, row[cap_tokens + 12: cap_tokens + 12 + micro], row[cap_tokens + 12 + micro:],
                                rate_d, ant.n_inst, ant.horizon, load, ovf, status)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        stage.copy_(rows_d[0])
        for _ in range(3):
            call_on_stage()                                                # first-call set-up happens outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call_on_stage()

    def replay(b):
        stage.copy_(rows_d[b])
        graph.replay()

    def run(issue, sync):
        lat, svc = np.zeros(total), np.zeros(total)
        t_start = time.perf_counter() + 0.01 - ready[0]
        for b in range(total):
            while True:
                now = time.perf_counter() - t_start
                if now >= ready[b]:
                    break
            issue(b)
            sync()
            done = time.perf_counter() - t_start
            lat[b], svc[b] = done - ready[b], done - now
        t = slice(warm, total)
        span = (ready[total - 1] + lat[total - 1]) - ready[warm]
        return {"p50_ms": 1e3 * float(np.quantile(lat[t], 0.5)), "p99_ms": 1e3 * float(np.quantile(lat[t], 0.99)),
                "mean_ms": 1e3 * float(lat[t].mean()), "service_p50_ms": 1e3 * float(np.quantile(svc[t], 0.5)),
                "service_p99_ms": 1e3 * float(np.quantile(svc[t], 0.99)),
                "requests_per_s": (n_batches - 1) * micro / span if n_batches > 1 else 0.0,
                "capacity_requests_per_s": micro / float(svc[t].mean())}

    out = {"workload": f"latency: 6-layer H768 A12 F3072 bf16 encoder, Poisson arrivals at {rate_per_s:.0f} requests/s in "
                       f"micro-batches of {micro} (lognormal(5.0,0.9) lengths in [4,512]); anticipator 4 x 64",
           "micro_batches": n_batches, "warmup_batches": warm, "tokens_per_batch_mean": float(lengths.sum()) / total,
           "eager": run(eager, torch.cuda.synchronize)}
    with torch.cuda.stream(side):
        out["graph"] = run(replay, side.synchronize)
    flags, _ = ps.ps_status_read(status)
    out["status_flags"] = int(flags)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="production", choices=sorted(WORKLOADS))
    ap.add_argument("--stream-records", type=int, default=44_100_000,
                    help="records of the anticipator bandwidth stream (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--latency-batches", type=int, default=2000,
                    help="timed micro-batches of the latency leg, after a tenth as many warm-up ones (0 = skip)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one plain elementwise copy of this many MiB (a known traffic for counter runs)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="instead of the benchmark: time the vendor library's bf16 GEMM (torch linear, bias only) on the "
                         "workload's four map shapes, as a yardstick for this library's GEMM kernel, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2504_03702_amd import binding as ps
    from paper_2504_03702_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 1
    ps.load_library()
    dev = torch.device("cuda:0")
    if args.copy_calibration > 0:
        # reads and writes exactly copy_calibration MiB: what FETCH_SIZE / WRITE_SIZE report for this
        # kernel scales the same counters of the other kernels in the run
        src = torch.ones(args.copy_calibration * 262144, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    model_kind, prompt_kind, ant_kind, desc = WORKLOADS[args.workload]
    cfg = wl.MODELS[model_kind].resolved()
    if args.vendor_gemm:
        # the rows one step's maps run over, random operands; the library's own kernel is chosen by torch
        rows = (int(wl.make_prompts(prompt_kind, seed=0).valid_lengths().sum()) + 255) // 256 * 256
        H, F = cfg.hidden, cfg.ffn
        res = []
        gen = torch.Generator(device=dev).manual_seed(0)
        for name, K, N in (("qkv", H, 3 * H), ("o_proj", H, H), ("ffn1", H, F), ("ffn2", F, H)):
            xa = torch.randn(rows, K, device=dev, generator=gen).to(torch.bfloat16)
            wb = (torch.randn(N, K, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
            bb = torch.zeros(N, device=dev, dtype=torch.bfloat16)
            for _ in range(2):
                torch.nn.functional.linear(xa, wb, bb)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                torch.nn.functional.linear(xa, wb, bb)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            res.append({"map": name, "rows": rows, "K": K, "N": N, "ms": ms, "TFLOP/s": 2.0 * rows * K * N / ms / 1e9})
            del xa, wb, bb
        print(json.dumps({"vendor_gemm": res, "workload": args.workload, "dtype": "bf16"}))
        return 0

    tmp = tempfile.mkdtemp(prefix="ps_bench_")
    model_path = os.path.join(tmp, f"{model_kind}.bin")
    wl.write_model(model_path, cfg, wl.make_weights(cfg, seed=0))
    model = ps.ps_model_load(model_path, 0)
    batch = wl.make_prompts(prompt_kind, seed=0)
    n_req = batch.n_req
    lengths = batch.valid_lengths()
    ant = wl.make_anticipator_inputs(ant_kind, seed=0, n=n_req, pred_tokens=np.zeros(n_req, np.int32))

    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    ids, offs = t32(batch.token_ids), t32(batch.offsets)
    lens = None if batch.lengths is None else t32(batch.lengths)
    inst, arr = t32(ant.instance_id), t32(ant.arrival_bucket)
    rate = None if ant.rate is None else t32(ant.rate)
    pred_f = torch.empty(n_req, dtype=torch.float32, device=dev)
    pred_t = torch.empty(n_req, dtype=torch.int32, device=dev)
    load = torch.zeros(ant.n_inst * ant.horizon, dtype=torch.int32, device=dev)
    ovf = torch.zeros(ant.n_inst, dtype=torch.int64, device=dev)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, ids.numel(), n_req), dev)
    aws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(n_req, ant.n_inst, ant.horizon), dev)
    status = ps.new_status(dev)

    # the same batch in the paper's own units: each request admitted into its instance's look-ahead map
    # with its prompt length and the prediction just made (Sec. 3.4.1)
    la = wl.make_lookahead_inputs(ant_kind if ant_kind in ("tiny", "production") else "medium", seed=0, n=n_req)
    la_start = t32(np.random.default_rng(7).integers(0, la.map_len // 4, n_req))
    la_prompt, la_zero = t32(lengths), torch.zeros(n_req, dtype=torch.int32, device=dev)
    la_sign = torch.ones(n_req, dtype=torch.int32, device=dev)
    la_inst = inst % la.n_inst
    la_kv = torch.zeros(la.n_inst * la.map_len, dtype=torch.int32, device=dev)
    la_ovf = torch.zeros(la.n_inst, dtype=torch.int64, device=dev)
    la_ws = ps.alloc_workspace(ps.ps_lookahead_workspace_bytes(n_req, la.n_inst, la.map_len), dev)

    def step():
        ps.ps_predict_load(model, ids, offs, lens, pred_f, pred_t, ws, status)
        ps.ps_anticipate(pred_t, inst, arr, rate, ant.n_inst, ant.horizon, load, ovf, aws, status)
        ps.ps_lookahead_update(la_inst, la_start, la_prompt, la_zero, pred_t, la_sign, la.n_inst, la.map_len,
                               la_kv, la_ovf, la_ws, status=status)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ps.ps_profile_enable(model, True)
    ps.ps_profile_read(model)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ps.ps_profile_read(model)
    core_ghz = ps.ps_profile_clock(model) if cfg.dtype == wl.DTYPE_BF16 else 0.0
    ps.ps_profile_enable(model, False)
    flags, _ = ps.ps_status_read(status)
    if flags:
        print(f"bench.py: device status flags {flags:#x}", file=sys.stderr)
        return 1
    ms_per_step = 1e3 * dt / args.steps

    # the two map updates of a step at the batch's own size are launch-latency bound: their time per call
    def call_us(fn, reps=50):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return 1e3 * a.elapsed_time(b) / reps
    ant_us = call_us(lambda: ps.ps_anticipate(pred_t, inst, arr, rate, ant.n_inst, ant.horizon, load, ovf, aws, status))
    la_us = call_us(lambda: ps.ps_lookahead_update(la_inst, la_start, la_prompt, la_zero, pred_t, la_sign, la.n_inst,
                                                   la.map_len, la_kv, la_ovf, la_ws, status=status))

    gemm_flops, attn_flops = encoder_flops(cfg, lengths)
    gemm_ms, gemm_launches = prof["gemm"]
    out = {
        "metric": "requests predicted/sec (1 GPU)", "value": n_req / (dt / args.steps), "unit": "requests/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == wl.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "requests": n_req, "tokens": int(lengths.sum()),
                   "algorithmic_tflop_per_step": (gemm_flops + attn_flops) / 1e12},
        "encoder_mfma_frac": (gemm_flops + attn_flops) / (dt / args.steps) / (PEAK_BF16_TFLOPS * 1e12),
        "kernel_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
        "map_updates_us_per_call": {"records": n_req, "anticipate": ant_us, "lookahead_update": la_us},
    }
    if cfg.dtype == wl.DTYPE_BF16 and gemm_launches:
        # dominant kernel: the bf16 MFMA GEMM (4 launches per layer); algorithmic flops per launch =
        # 2*K*N flops per token row, i.e. (8 H^2 + 4 H F) per token per layer over its 4 launches
        per_launch_flops = gemm_flops * args.steps / gemm_launches
        per_launch_s = gemm_ms * 1e-3 / gemm_launches
        achieved = per_launch_flops / per_launch_s / 1e12
        out["roofline"] = {"bound": "mfma", "kernel": "gemm_bf16_kernel", "achieved": achieved,
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                           "traffic": measured_gemm_traffic(args.workload), "launches_per_step": gemm_launches // args.steps,
                           "avg_launch_ms": 1e3 * per_launch_s}
        # algorithmic bytes of the same average launch: activations in, weights once, outputs (and the
        # fp32 residual sums in and out for the two launches that carry them)
        H, F, T, L = cfg.hidden, cfg.ffn, int(lengths.sum()), cfg.layers
        qkv_b = T * (2 * H + 6 * H) + 6 * H * H
        rest_b = T * (2 * H + 8 * H) + T * (2 * H + 2 * F) + T * (2 * F + 8 * H) + 2 * H * H + 4 * H * F
        kv_b = T * (2 * H + 4 * H) + 4 * H * H                  # last layer: keys and values only
        out["roofline"]["algorithmic_bytes"] = ((L - 1) * (qkv_b + rest_b) + kv_b) / (4 * (L - 1) + 1)
        if core_ghz > 0:
            # the core clock the chip sustained inside the last GEMM launch (the published peak assumes
            # 2.4 GHz): achieved / (peak * clock / 2.4) is the matrix cores' utilisation at that clock
            out["roofline"]["core_clock_ghz_in_kernel"] = core_ghz
            out["roofline"]["frac_at_sustained_clock"] = achieved / (PEAK_BF16_TFLOPS * core_ghz / 2.4)
        att_ms = prof["attention"][0]
        if att_ms > 0:
            out["attention_tflops"] = attn_flops * args.steps / (att_ms * 1e-3) / 1e12

    # ---- anticipator on a long record stream (the call sizes above are launch-latency bound) ----
    if args.stream_records > 0:
        del ws
        torch.cuda.empty_cache()
        # two orders of the same record stream: arrival buckets independent of position (the headline figure)
        # and as a request log (the same records in arrival order, which the library exploits)
        for key, kind in (("anticipator", "stream"), ("anticipator_by_arrival", "stream_by_arrival")):
            s_in = wl.make_anticipator_inputs(kind, seed=0, n=args.stream_records)
            sp, si, sa, sr = t32(s_in.pred_tokens), t32(s_in.instance_id), t32(s_in.arrival_bucket), t32(s_in.rate)
            sload = torch.zeros(s_in.n_inst * s_in.horizon, dtype=torch.int32, device=dev)
            sovf = torch.zeros(s_in.n_inst, dtype=torch.int64, device=dev)
            sws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(args.stream_records, s_in.n_inst, s_in.horizon), dev)
            reps = 10
            for _ in range(2):
                ps.ps_anticipate(sp, si, sa, sr, s_in.n_inst, s_in.horizon, sload, sovf, sws, status)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                ps.ps_anticipate(sp, si, sa, sr, s_in.n_inst, s_in.horizon, sload, sovf, sws, status)
            e1.record()
            torch.cuda.synchronize()
            call_s = e0.elapsed_time(e1) * 1e-3 / reps
            # algorithmic bytes: three int32 per record read, the map read and written once
            nbytes = 12.0 * args.stream_records + 8.0 * s_in.n_inst * s_in.horizon
            gbs = nbytes / call_s / 1e9
            out[key] = {"bound": "hbm", "records": args.stream_records, "order": kind, "ms_per_call": 1e3 * call_s,
                        "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                        "records_per_s": args.stream_records / call_s}
            del sp, si, sa, sr, sload, sovf, sws
        # how the rate builds up with the record count (arbitrary order)
        ramp = []
        for n_r in (1 << 20, 1 << 24):
            if n_r >= args.stream_records:
                continue
            r_in = wl.make_anticipator_inputs("stream", seed=0, n=n_r)
            rp, ri, ra, rr = t32(r_in.pred_tokens), t32(r_in.instance_id), t32(r_in.arrival_bucket), t32(r_in.rate)
            rload = torch.zeros(r_in.n_inst * r_in.horizon, dtype=torch.int32, device=dev)
            rovf = torch.zeros(r_in.n_inst, dtype=torch.int64, device=dev)
            rws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(n_r, r_in.n_inst, r_in.horizon), dev)
            for _ in range(2):
                ps.ps_anticipate(rp, ri, ra, rr, r_in.n_inst, r_in.horizon, rload, rovf, rws, status)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                ps.ps_anticipate(rp, ri, ra, rr, r_in.n_inst, r_in.horizon, rload, rovf, rws, status)
            e1.record()
            torch.cuda.synchronize()
            r_s = e0.elapsed_time(e1) * 1e-3 / 20
            ramp.append({"records": n_r, "ms_per_call": 1e3 * r_s,
                         "GB/s": (12.0 * n_r + 8.0 * r_in.n_inst * r_in.horizon) / r_s / 1e9})
            del rp, ri, ra, rr, rload, rovf, rws
        out["anticipator"]["ramp"] = ramp
        # yardstick: a kernel that only reads a buffer of the stream's size (three int32 per record)
        buf = torch.randint(0, 1 << 30, (3 * ((args.stream_records + 3) // 4 * 4),), dtype=torch.int32, device=dev)
        sink = torch.zeros(1, dtype=torch.int64, device=dev)
        for _ in range(2):
            ps.ps_profile_stream_read(buf, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            ps.ps_profile_stream_read(buf, sink)
        e1.record()
        torch.cuda.synchronize()
        rd_s = e0.elapsed_time(e1) * 1e-3 / 10
        rd_gbs = buf.numel() * 4 / rd_s / 1e9
        out["stream_read_yardstick"] = {"bytes": buf.numel() * 4, "ms_per_call": 1e3 * rd_s, "GB/s": rd_gbs,
                                        "frac_of_peak": rd_gbs / PEAK_HBM_GBS}
        for key in ("anticipator", "anticipator_by_arrival"):
            out[key]["frac_of_read_only_kernel"] = out[key]["achieved"] / rd_gbs
        del buf, sink

    # ---- look-ahead map in KV-token units on a long record stream -----------------------------------
    if args.stream_records > 0:
        torch.cuda.empty_cache()
        n_la = min(args.stream_records, 10_000_000)
        s_la = wl.make_lookahead_inputs("stream", seed=0, n=n_la)
        cols = [t32(c) for c in s_la.columns()]
        n_rec = cols[0].numel()
        kv = torch.zeros(s_la.n_inst * s_la.map_len, dtype=torch.int32, device=dev)
        ovf2 = torch.zeros(s_la.n_inst, dtype=torch.int64, device=dev)
        lws = ps.alloc_workspace(ps.ps_lookahead_workspace_bytes(n_rec, s_la.n_inst, s_la.map_len), dev)
        reps = 10
        for _ in range(2):
            ps.ps_lookahead_update(*cols, s_la.n_inst, s_la.map_len, kv, ovf2, lws, status=status)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            ps.ps_lookahead_update(*cols, s_la.n_inst, s_la.map_len, kv, ovf2, lws, status=status)
        e1.record()
        torch.cuda.synchronize()
        call_s = e0.elapsed_time(e1) * 1e-3 / reps
        # algorithmic bytes: six int32 per record read, the int32 map read and written once
        nbytes = 24.0 * n_rec + 8.0 * s_la.n_inst * s_la.map_len
        gbs = nbytes / call_s / 1e9
        out["lookahead"] = {"bound": "hbm", "records": n_rec, "ms_per_call": 1e3 * call_s, "achieved": gbs,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                            "records_per_s": n_rec / call_s}
        del cols, kv, lws

    # ---- router scoring over the production micro-batch (sequential by definition: one workgroup) ----
    if args.stream_records > 0:
        K_r, l_r = 256, 100
        rng = np.random.default_rng(11)
        cap_r = t32(rng.integers(120_000, 400_001, K_r))
        win0 = t32(rng.integers(0, 100_000, K_r * l_r))
        q0 = torch.from_numpy(rng.integers(0, 3000, K_r).astype(np.int64)).to(dev)
        d0 = torch.from_numpy(rng.integers(0, 20000, K_r).astype(np.int64)).to(dev)
        asg = torch.empty(n_req, dtype=torch.int32, device=dev)
        sc = torch.empty(n_req, dtype=torch.int64, device=dev)
        reps = 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(reps + 1):
            if i == 1:
                e0.record()
            ps.ps_route(la_prompt, pred_t, K_r, l_r, win0.clone(), cap_r, q0.clone(), d0.clone(), asg, sc, status=status)
        e1.record()
        torch.cuda.synchronize()
        route_s = e0.elapsed_time(e1) * 1e-3 / reps
        out["router"] = {"requests": n_req, "instances": K_r, "window": l_r, "ms_per_batch": 1e3 * route_s,
                         "requests_per_s": n_req / route_s, "us_per_request": 1e6 * route_s / n_req}

    # ---- scaler's checks over every instance's map, and the service workload forecasts (both small) ----
    if args.stream_records > 0:
        def timed(fn, reps=20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        K_s, L_s, win_s = 256, 4096, 100
        rng = np.random.default_rng(12)
        kv_s = t32(rng.integers(0, 400_000, K_s * L_s))
        cap_s = t32(rng.integers(120_000, 400_001, K_s))
        i32 = lambda n_: torch.empty(n_, dtype=torch.int32, device=dev)
        oc, pk, ov, sm = i32(K_s), i32(K_s), i32(K_s), i32(2)
        sd = torch.empty(1, dtype=torch.float64, device=dev)
        scan_s = timed(lambda: ps.ps_scaler_scan(kv_s, cap_s, K_s, L_s, win_s, oc, pk, ov, sm, sd))
        out["scaler"] = {"instances": K_s, "map_len": L_s, "window": win_s, "us_per_scan": 1e6 * scan_s}
        fc = wl.make_forecaster_inputs(seed=0, n_services=512, hidden=64, k=24)
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32).reshape(-1)).to(dev)
        fw, fp, fd, fm = f32(fc.weights), f32(fc.hist_p), f32(fc.hist_d), f32(fc.mu)
        fo = torch.empty(512 * 5, dtype=torch.float32, device=dev)
        fc_s = timed(lambda: ps.ps_forecast(fw, 64, fp, fd, 512, 24, fm, fo))
        out["forecaster"] = {"services": 512, "hidden": 64, "history": 24, "us_per_call": 1e6 * fc_s}

    if args.latency_batches > 0:
        torch.cuda.empty_cache()
        out["latency"] = latency_leg(torch, ps, wl, dev, status, args.latency_batches, max(1, args.latency_batches // 10))

    if not args.no_cpu_baseline:
        stream = wl.make_anticipator_inputs("stream", seed=0, n=args.stream_records) if args.stream_records > 0 else None
        out["cpu_baseline"] = time_cpu_oracle(model_path, batch, ant, stream)
    try:
        os.remove(model_path)
        os.rmdir(tmp)
    except OSError:
        pass
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
