"""GPU parity of ps_predict_load (bf16 models: MFMA GEMMs, MFMA attention) against the fp64
oracle on the same seeded inputs, through the C ABI."""
import dataclasses
import os

import numpy as np
import pytest

from oracle import predictor as op
from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
from oracle import pool as oracle_pool
from tests.gpu_util import TOL_BF16, rel_err, run_predict

pytestmark = pytest.mark.gpu

# a small encoder with the bf16 path's shape constraints (hidden, ffn multiples of 256; head size 64)
SMALL = wl.ModelConfig(layers=2, hidden=256, heads=4, ffn=512, vocab=1000, max_pos=640, dtype=wl.DTYPE_BF16)


def make(tmp_models, name, cfg, **kw):
    path = os.path.join(tmp_models, name)
    if not os.path.exists(path):
        wl.write_model(path, cfg, wl.make_weights(cfg, seed=0, **kw))
    return ps.ps_model_load(path, 0), op.load_model(path)


def check(model, ref, batch, tol=TOL_BF16):
    got_f, got_t, flags, _ = run_predict(model, batch)
    ref_f, ref_t = op.predict_load(ref, batch.token_ids, batch.offsets, batch.lengths)
    assert flags == 0
    err = rel_err(got_f, ref_f)
    print(f"  max rel err {err.max():.3e}  mean {err.mean():.3e}  spread of oracle {np.std(ref_f):.2f}", flush=True)
    assert err.max() < tol
    d_max = model.info.d_max
    assert np.array_equal(got_t, np.clip(np.rint(got_f.astype(np.float32)), 0, d_max).astype(np.int32))
    # the integer decision is taken in the kernel's precision; it can differ from the oracle's by the
    # float tolerance, rounded up, plus one for the rounding itself
    slack = np.ceil(tol * np.maximum(np.abs(ref_f), np.sqrt(np.mean(ref_f ** 2)))) + 1
    assert np.all(np.abs(got_t - ref_t) <= slack)
    return got_f


@pytest.mark.parametrize("lengths", [
    [1], [64], [65], [128], [129], [3, 640, 1, 130, 64, 257],
    list(range(1, 40)),                       # many short requests: row alignment gaps everywhere
    [500, 377, 256, 255, 128, 127, 63, 600],  # several key tiles, ragged tails, > 256 rows per request
])
def test_small_model_shapes(tmp_models, lengths):
    print(f"predict bf16 small lengths={lengths[:8]}", flush=True)
    model, ref = make(tmp_models, "small_bf16.bin", SMALL, ln_jitter=0.1, bias_std=0.05)
    rng = np.random.default_rng(len(lengths))
    lengths = np.array(lengths, np.int32)
    batch = wl.pack_prompts(lengths, rng.integers(0, SMALL.vocab, int(lengths.sum())).astype(np.int32))
    check(model, ref, batch)


def test_single_layer_model(tmp_models):
    """One layer: the first layer is also the last, where only the requests' first rows go on."""
    cfg = dataclasses.replace(SMALL, layers=1)
    model, ref = make(tmp_models, "small_bf16_1layer.bin", cfg, ln_jitter=0.1, bias_std=0.05)
    lengths = np.array([1, 33, 64, 200, 129, 7], np.int32)
    ids = np.random.default_rng(5).integers(0, cfg.vocab, int(lengths.sum())).astype(np.int32)
    check(model, ref, wl.pack_prompts(lengths, ids))


def test_widest_model(tmp_models):
    """hidden = 2048, the widest the bf16 kernels accept: 32 heads, 8 tile columns in the hidden-wide maps,
    32 partial row sums per row; LayerNorm scale and shift well away from 1 and 0 (they are folded into
    the weights of the following map), a mean offset in the residual stream through the biases."""
    cfg = wl.ModelConfig(layers=3, hidden=2048, heads=32, ffn=512, vocab=500, max_pos=300, head_hidden=64,
                         dtype=wl.DTYPE_BF16)
    model, ref = make(tmp_models, "wide_bf16.bin", cfg, ln_jitter=0.3, bias_std=0.2)
    lengths = np.array([5, 257, 64, 130], np.int32)
    ids = np.random.default_rng(8).integers(0, cfg.vocab, int(lengths.sum())).astype(np.int32)
    print("predict bf16 hidden 2048", flush=True)
    check(model, ref, wl.pack_prompts(lengths, ids))


def test_profile_hooks(tmp_models):
    """Kernel-family timing and the clock probe: plausible values, nothing left behind when off."""
    model, _ = make(tmp_models, "small_bf16.bin", SMALL, ln_jitter=0.1, bias_std=0.05)
    lengths = np.full(64, 512, np.int32)
    ids = np.random.default_rng(6).integers(0, SMALL.vocab, int(lengths.sum())).astype(np.int32)
    batch = wl.pack_prompts(lengths, ids)
    ps.ps_profile_enable(model, True)
    ps.ps_profile_read(model)
    run_predict(model, batch)
    prof = ps.ps_profile_read(model)
    ghz = ps.ps_profile_clock(model)
    ps.ps_profile_enable(model, False)
    assert set(prof) == set(ps.PS_FAMILIES)
    assert prof["gemm"][1] == 4 * (SMALL.layers - 1) + 1 and prof["gemm"][0] > 0
    assert prof["attention"][1] == SMALL.layers and prof["head"][1] == 1
    assert 0.3 < ghz < 3.0
    run_predict(model, batch)
    assert all(v == (0.0, 0) for v in ps.ps_profile_read(model).values())


def test_padded_equals_packed_and_learnable_prompts(tmp_models):
    cfg = dataclasses.replace(SMALL, n_soft=5, layers=3)
    model, ref = make(tmp_models, "small_bf16_soft.bin", cfg, ln_jitter=0.1, bias_std=0.05)
    rng = np.random.default_rng(11)
    lengths = np.array([17, 300, 1, 64, 59, 123, 635], np.int32)
    ids = rng.integers(0, cfg.vocab, int(lengths.sum())).astype(np.int32)
    packed, padded = wl.pack_prompts(lengths, ids), wl.pad_prompts(lengths, ids, pad_id=3)
    a = check(model, ref, packed)
    b = check(model, ref, padded)
    assert np.array_equal(a, b)              # padding is compacted away: same rows, same arithmetic


def test_bert_base_padded_batch(tmp_models):
    """BERT-base-shaped encoder, 64 prompts padded to the batch maximum."""
    print("predict bf16 bert_base padded 64", flush=True)
    cfg = wl.MODELS["bert_base"]
    model, ref = make(tmp_models, "bert_base.bin", cfg)
    batch = wl.make_prompts("bert_base_padded", seed=0)
    check(model, ref, batch)


def requests_of(batch, picks):
    return [batch.token_ids[batch.offsets[r]:batch.offsets[r + 1]] for r in picks]


def stratified(lengths, candidates, count):
    """`count` of the candidate requests spread evenly over their length ranks (shortest and longest included)."""
    by_len = candidates[np.argsort(lengths[candidates], kind="stable")]
    return by_len[np.unique(np.linspace(0, len(by_len) - 1, count).round().astype(np.int64))]


def check_against_pool(tag, model_path, batch, got_f, got_t, picks, d_max):
    """Oracle (one request at a time, on the host's cores) against the GPU's predictions for `picks`."""
    ref_f = oracle_pool.predict_requests(model_path, requests_of(batch, picks))
    # the scale of the tolerance is the batch's RMS; the RMS over these hundreds of requests stands in for it
    scale = np.maximum(np.abs(ref_f), np.sqrt(np.mean(ref_f ** 2)))
    err = np.abs(got_f[picks] - ref_f) / scale
    worst = int(np.argmax(err))
    lengths = batch.valid_lengths()
    print(f"  {tag}: {len(picks)} requests, {int(lengths[picks].sum())} tokens: max rel err {err.max():.3e} "
          f"(request {int(picks[worst])}, {int(lengths[picks[worst]])} tokens), p99 {np.quantile(err, 0.99):.3e}, "
          f"mean {err.mean():.3e}", flush=True)
    assert err.max() < TOL_BF16
    ref_t = np.clip(np.rint(ref_f), 0, d_max).astype(np.int32)
    assert np.all(np.abs(got_t[picks] - ref_t) <= np.ceil(TOL_BF16 * scale) + 1)


def chunks_bit_equal(model, batch, got_f, got_t, chunk=256):
    """The same requests in calls of `chunk` requests each (other row counts, other tile walks): bit-equal."""
    lengths = batch.valid_lengths()
    for r0 in range(0, batch.n_req, chunk):
        picks = np.arange(r0, min(r0 + chunk, batch.n_req))
        sub = wl.pack_prompts(lengths[picks], np.concatenate(requests_of(batch, picks)))
        f, t, flags, _ = run_predict(model, sub)
        assert flags == 0 and np.array_equal(f, got_f[picks]) and np.array_equal(t, got_t[picks]), f"chunk at {r0}"


@pytest.fixture(scope="module")
def bert_varlen(tmp_models):
    cfg = wl.MODELS["bert_base"]
    model, _ = make(tmp_models, "bert_base.bin", cfg)
    batch = wl.make_prompts("bert_base_varlen", seed=0)
    got_f, got_t, flags, _ = run_predict(model, batch)
    assert flags == 0 and np.isfinite(got_f).all()
    return model, os.path.join(tmp_models, "bert_base.bin"), batch, got_f, got_t


def test_bert_base_varlen_chunks_bit_equal(bert_varlen):
    """The 1024-prompt packed batch runs whole on the GPU; the same requests in four calls of 256 give the same
    bits (a request's prediction does not depend on the rest of the batch, nor on where its rows fall)."""
    print("predict bf16 bert_base varlen 1024: whole batch against chunks of 256", flush=True)
    model, _, batch, got_f, got_t = bert_varlen
    chunks_bit_equal(model, batch, got_f, got_t)


def test_bert_base_varlen_against_oracle(bert_varlen):
    """Every request of at most 48 tokens (short prompts carry the largest errors) and 64 others spread evenly
    over the length ranks, each against the oracle."""
    print("predict bf16 bert_base varlen 1024: short prompts and a length-stratified sample against the oracle", flush=True)
    model, path, batch, got_f, got_t = bert_varlen
    lengths = batch.valid_lengths()
    short = np.flatnonzero(lengths <= 48)
    rest = stratified(lengths, np.flatnonzero(lengths > 48), 64)
    check_against_pool("short + stratified", path, batch, got_f, got_t, np.concatenate([short, rest]), model.info.d_max)


def test_latency_shape_micro_batches(tmp_models):
    """6-layer DistilBERT-shaped encoder on micro-batches of 8 prompts."""
    print("predict bf16 latency micro-batches", flush=True)
    cfg = wl.MODELS["latency"]
    model, ref = make(tmp_models, "latency.bin", cfg)
    for seed in (0, 1):
        check(model, ref, wl.make_prompts("latency", seed=seed))


@pytest.fixture(scope="module")
def production(tmp_models):
    """The benchmark's own launch configuration: 16-layer H1024 encoder, 4096 packed prompts up to 2048 tokens,
    then ps_anticipate over 256 x 600 on the predictions, same stream."""
    import torch
    cfg = wl.MODELS["production"]
    model, _ = make(tmp_models, "production.bin", cfg)
    batch = wl.make_prompts("production", seed=0)
    n = batch.n_req
    dev = "cuda:0"
    ids = torch.from_numpy(batch.token_ids).to(dev)
    offs = torch.from_numpy(batch.offsets).to(dev)
    pred_f = torch.empty(n, dtype=torch.float32, device=dev)
    pred_t = torch.empty(n, dtype=torch.int32, device=dev)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, ids.numel(), n), dev)
    ant = wl.make_anticipator_inputs("production", seed=0, n=n, pred_tokens=np.zeros(n, np.int32))
    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(dev)
    inst, arr, rate = t32(ant.instance_id), t32(ant.arrival_bucket), t32(ant.rate)
    load = torch.zeros(ant.n_inst * ant.horizon, dtype=torch.int32, device=dev)
    ovf = torch.zeros(ant.n_inst, dtype=torch.int64, device=dev)
    aws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(n, ant.n_inst, ant.horizon), dev)
    st = ps.new_status(dev)
    ps.ps_predict_load(model, ids, offs, None, pred_f, pred_t, ws, st)
    ps.ps_anticipate(pred_t, inst, arr, rate, ant.n_inst, ant.horizon, load, ovf, aws, st)
    flags, _ = ps.ps_status_read(st)
    assert flags == 0
    return dict(model=model, path=os.path.join(tmp_models, "production.bin"), batch=batch, ant=ant,
                got_f=pred_f.cpu().numpy(), got_t=pred_t.cpu().numpy(),
                load=load.cpu().numpy().reshape(ant.n_inst, ant.horizon), ovf=ovf.cpu().numpy())


def test_production_batch_fused_anticipator(production):
    """The histograms are bit-exact against the oracle fed the GPU's own integer predictions, and the totals
    invariant holds on everything."""
    from oracle import anticipator as oa
    print("predict bf16 production 4096 + anticipator", flush=True)
    p = production
    got_f, got_t, ant = p["got_f"], p["got_t"], p["ant"]
    assert np.isfinite(got_f).all()
    assert np.array_equal(got_t, np.clip(np.rint(got_f), 0, p["model"].info.d_max).astype(np.int32))
    ref_load, ref_ovf, status, _ = oa.anticipate(got_t, ant.instance_id, ant.arrival_bucket, ant.rate,
                                                 ant.n_inst, ant.horizon)
    assert status == 0 and np.array_equal(p["load"], ref_load) and np.array_equal(p["ovf"], ref_ovf)
    per_inst = np.bincount(ant.instance_id, weights=got_t, minlength=ant.n_inst).astype(np.int64)
    assert np.array_equal(p["load"].sum(axis=1, dtype=np.int64) + p["ovf"], per_inst)


def test_production_batch_chunks_bit_equal(production):
    """All 4096 requests again in 16 calls of 256: the same bits as in the one call the benchmark times."""
    print("predict bf16 production 4096: whole batch against chunks of 256", flush=True)
    p = production
    chunks_bit_equal(p["model"], p["batch"], p["got_f"], p["got_t"])


def test_production_short_prompts_against_oracle(production):
    """Every request of at most 48 tokens (366 of the 4096; short prompts carry the largest errors: few keys
    to average the operands' rounding over) against the oracle."""
    print("predict bf16 production 4096: every prompt of at most 48 tokens against the oracle", flush=True)
    p = production
    lengths = p["batch"].valid_lengths()
    short = np.flatnonzero(lengths <= 48)
    assert len(short) >= 300
    check_against_pool("short prompts", p["path"], p["batch"], p["got_f"], p["got_t"], short, p["model"].info.d_max)


def test_production_stratified_sample_against_oracle(production):
    """72 longer requests spread evenly over the length ranks (49 to 2048 tokens, the longest included), the
    first and the last request of the batch: each against the oracle."""
    print("predict bf16 production 4096: length-stratified sample against the oracle", flush=True)
    p = production
    lengths = p["batch"].valid_lengths()
    rest = stratified(lengths, np.flatnonzero(lengths > 48), 72)
    picks = np.unique(np.concatenate([rest, [0, p["batch"].n_req - 1, int(np.argmax(lengths))]]))
    picks = picks[lengths[picks] > 48]
    check_against_pool("stratified", p["path"], p["batch"], p["got_f"], p["got_t"], picks, p["model"].info.d_max)
