"""GPU parity of ps_predict_load (bf16 models: MFMA GEMMs, MFMA attention) against the fp64
oracle on the same seeded inputs, through the C ABI."""
import dataclasses
import os

import numpy as np
import pytest

from oracle import predictor as op
from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
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


def test_bert_base_varlen_sampled(tmp_models):
    """The 1024-prompt packed batch runs whole on the GPU; the oracle checks a sample of requests
    (a request's prediction does not depend on the rest of the batch)."""
    print("predict bf16 bert_base varlen 1024", flush=True)
    cfg = wl.MODELS["bert_base"]
    model, ref = make(tmp_models, "bert_base.bin", cfg)
    batch = wl.make_prompts("bert_base_varlen", seed=0)
    got_f, got_t, flags, _ = run_predict(model, batch)
    assert flags == 0 and np.isfinite(got_f).all()
    lengths = batch.valid_lengths()
    pick = np.unique(np.concatenate([[0, 1023, int(np.argmax(lengths)), int(np.argmin(lengths))],
                                     np.random.default_rng(0).choice(1024, 20, replace=False)]))
    sub = wl.pack_prompts(lengths[pick], np.concatenate([batch.token_ids[batch.offsets[r]:batch.offsets[r + 1]] for r in pick]))
    ref_f, _ = op.predict_load(ref, sub.token_ids, sub.offsets)
    scale = np.maximum(np.abs(ref_f), np.sqrt(np.mean(ref_f ** 2)))
    err = np.abs(got_f[pick] - ref_f) / scale
    print(f"  max rel err {err.max():.3e} mean {err.mean():.3e}", flush=True)
    assert err.max() < TOL_BF16
    # the same requests alone give bit-identical results: no cross-request leakage
    alone_f, _, _, _ = run_predict(model, sub)
    assert np.array_equal(alone_f, got_f[pick])
