"""GPU parity of ps_predict_load (fp32 models) against the fp64 oracle, through the C ABI."""
import dataclasses
import os

import numpy as np
import pytest

from oracle import predictor as op
from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
from tests.gpu_util import TOL_FP32, rel_err, run_predict

pytestmark = pytest.mark.gpu
TINY = wl.MODELS["tiny"]


def make(tmp_models, name, cfg=TINY, **kw):
    path = os.path.join(tmp_models, name)
    wl.write_model(path, cfg, wl.make_weights(cfg, seed=0, **kw))
    return ps.ps_model_load(path, 0), op.load_model(path)


def check_tokens(got_f, got_t, ref_t, d_max, tol_tokens=1):
    # the rounding decision is taken in the kernel's precision (fp32) on the kernel's own value
    assert np.array_equal(got_t, np.clip(np.rint(got_f.astype(np.float32)), 0, d_max).astype(np.int32))
    assert np.max(np.abs(got_t - ref_t)) <= tol_tokens


@pytest.mark.parametrize("seed,n_req", [(0, 16), (1, 1), (2, 7), (3, 300)])
def test_tiny_config(tmp_models, seed, n_req):
    print(f"predict fp32 tiny seed={seed} n_req={n_req}", flush=True)
    model, ref = make(tmp_models, "tiny_gpu.bin", ln_jitter=0.1 if seed else 0.0, bias_std=0.05 if seed else 0.0)
    batch = wl.make_prompts("tiny", seed, n_req=n_req)
    got_f, got_t, flags, _ = run_predict(model, batch)
    ref_f, ref_t = op.predict_load(ref, batch.token_ids, batch.offsets)
    assert flags == 0
    assert rel_err(got_f, ref_f).max() < TOL_FP32
    check_tokens(got_f, got_t, ref_t, TINY.d_max)
    assert n_req == 1 or np.ptp(ref_f) > 1.0


def test_padded_layout_equals_packed(tmp_models):
    model, ref = make(tmp_models, "tiny_gpu.bin")
    packed = wl.make_prompts("tiny", 5, n_req=9)
    padded = wl.pad_prompts(packed.valid_lengths(), packed.token_ids, pad_id=77)
    a_f, a_t, fa, _ = run_predict(model, packed)
    b_f, b_t, fb, _ = run_predict(model, padded)
    assert fa == 0 and fb == 0
    assert np.array_equal(a_f, b_f) and np.array_equal(a_t, b_t)       # same rows, same arithmetic
    ref_f, _ = op.predict_load(ref, padded.token_ids, padded.offsets, padded.lengths)
    assert rel_err(b_f, ref_f).max() < TOL_FP32


def test_learnable_prompts_and_odd_shapes(tmp_models):
    # M = 4 learnable prompt rows; 3 heads of size 20; widths that are no multiple of a tile
    cfg = wl.ModelConfig(layers=3, hidden=60, heads=3, ffn=100, vocab=500, max_pos=80, n_soft=4,
                         head_hidden=33, dtype=wl.DTYPE_FP32)
    model, ref = make(tmp_models, "odd_soft.bin", cfg=cfg, ln_jitter=0.1, bias_std=0.05)
    rng = np.random.default_rng(7)
    lengths = np.array([1, 76, 2, 33, 64, 5], np.int32)
    batch = wl.pack_prompts(lengths, rng.integers(0, cfg.vocab, int(lengths.sum())).astype(np.int32))
    got_f, got_t, flags, _ = run_predict(model, batch)
    ref_f, ref_t = op.predict_load(ref, batch.token_ids, batch.offsets)
    assert flags == 0
    assert rel_err(got_f, ref_f).max() < TOL_FP32
    check_tokens(got_f, got_t, ref_t, cfg.d_max)


def test_batch_order_invariance(tmp_models):
    model, _ = make(tmp_models, "tiny_gpu.bin")
    b = wl.make_prompts("tiny", 6, n_req=8)
    lengths = b.valid_lengths()
    chunks = [b.token_ids[b.offsets[r]:b.offsets[r + 1]] for r in range(8)]
    perm = np.array([5, 2, 7, 0, 3, 6, 1, 4])
    pb = wl.pack_prompts(lengths[perm], np.concatenate([chunks[r] for r in perm]))
    a_f, _, _, _ = run_predict(model, b)
    p_f, _, _, _ = run_predict(model, pb)
    assert np.array_equal(p_f, a_f[perm])


def test_faulty_requests_are_isolated(tmp_models):
    model, ref = make(tmp_models, "tiny_gpu.bin")
    b = wl.make_prompts("tiny", 8, n_req=6)
    good_f, good_t, _, _ = run_predict(model, b)
    ids = b.token_ids.copy()
    ids[b.offsets[2] + 3] = TINY.vocab            # request 2: token id out of range
    ids[b.offsets[4]] = -1                        # request 4: negative id
    bad = dataclasses.replace(b, token_ids=ids)
    f, t, flags, first = run_predict(model, bad)
    assert flags == ps.PS_ST_BAD_TOKEN and first == 2
    assert np.isnan(f[[2, 4]]).all() and (t[[2, 4]] == -1).all()
    keep = [0, 1, 3, 5]
    assert np.array_equal(f[keep], good_f[keep]) and np.array_equal(t[keep], good_t[keep])
    with pytest.raises(op.OracleError):
        op.predict_load(ref, ids, b.offsets)
    # lengths: zero, longer than the span, longer than the position table
    padded = wl.pad_prompts(b.valid_lengths(), b.token_ids)
    lens = padded.lengths.copy()
    lens[1] = 0
    lens[3] = int(np.diff(padded.offsets)[3]) + 1
    f, t, flags, first = run_predict(model, dataclasses.replace(padded, lengths=lens))
    assert flags == ps.PS_ST_BAD_LENGTH and first == 1
    assert np.isnan(f[[1, 3]]).all() and (t[[1, 3]] == -1).all()
    assert np.array_equal(f[[0, 2, 4, 5]], good_f[[0, 2, 4, 5]])
    long_ids = np.zeros(TINY.max_pos + 1, np.int32)
    f, t, flags, _ = run_predict(model, wl.pack_prompts(np.array([TINY.max_pos + 1]), long_ids))
    assert flags == ps.PS_ST_BAD_LENGTH and np.isnan(f[0]) and t[0] == -1


def test_wrong_offsets_are_rejected_on_the_device(tmp_models):
    """Offsets are device data: spans that leave the token array, run backwards or overlap so that
    together they ask for more rows than the workspace was sized for are flagged, their requests get
    NaN / -1, and nothing is read or written out of bounds.  All buffers have the sizes the call states."""
    model, _ = make(tmp_models, "tiny_gpu.bin")
    b = wl.make_prompts("tiny", 8, n_req=6)
    good_f, good_t, _, _ = run_predict(model, b)
    n_tok = int(b.offsets[-1])
    # request 1 starts before the array, request 4 ends after it
    offs = b.offsets.copy()
    offs[1] = -3
    f, t, flags, first = run_predict(model, dataclasses.replace(b, offsets=offs))
    assert flags == ps.PS_ST_BAD_LENGTH and first == 0        # span 0 ends at -3 < its start
    assert np.isnan(f[[0, 1]]).all() and (t[[0, 1]] == -1).all()
    assert np.array_equal(f[2:], good_f[2:])
    offs = b.offsets.copy()
    offs[5] = n_tok + 40                                       # request 4 runs past the end, request 5 starts there
    f, t, flags, first = run_predict(model, dataclasses.replace(b, offsets=offs))
    assert flags == ps.PS_ST_BAD_LENGTH and first == 4
    assert np.isnan(f[[4, 5]]).all() and np.array_equal(f[:4], good_f[:4])
    # offsets 0, span, 0, span, ...: every even request claims the same valid span [0, span), every odd one runs
    # backwards.  Each even request is valid on its own; together they need several times the rows the host
    # planned for from the size of the token array
    import torch
    span = min(TINY.max_pos, n_tok)
    n_req = 40
    offs = np.tile(np.array([0, span], np.int32), n_req)[: n_req + 1].copy()
    dev = "cuda:0"
    ids = torch.from_numpy(b.token_ids).to(dev)
    pf = torch.full((n_req,), 5.0, dtype=torch.float32, device=dev)
    pt = torch.full((n_req,), -7, dtype=torch.int32, device=dev)
    ws = ps.alloc_workspace(ps.ps_workspace_bytes(model, n_tok, n_req), dev)
    st = ps.new_status(dev)
    ps.ps_predict_load(model, ids, torch.from_numpy(offs).to(dev), None, pf, pt, ws, st)
    flags, first = ps.ps_status_read(st)
    f, t = pf.cpu().numpy(), pt.cpu().numpy()
    assert flags == ps.PS_ST_BAD_LENGTH and first == 1
    assert np.isnan(f[1::2]).all() and (t[1::2] == -1).all()
    even = f[0::2]
    n_ok = int(np.sum(~np.isnan(even)))
    assert 1 <= n_ok < even.size and not np.isnan(even[:n_ok]).any() and np.isnan(even[n_ok:]).all()
    assert np.all(even[:n_ok] == even[0])                      # the same prompt every time
    assert (t[0::2][n_ok:] == -1).all()


def test_host_side_argument_errors(tmp_models):
    import torch
    model, _ = make(tmp_models, "tiny_gpu.bin")
    b = wl.make_prompts("tiny", 0, n_req=4)
    dev = "cuda:0"
    ids = torch.from_numpy(b.token_ids).to(dev)
    offs = torch.from_numpy(b.offsets).to(dev)
    pf = torch.empty(4, dtype=torch.float32, device=dev)
    pt = torch.empty(4, dtype=torch.int32, device=dev)
    with pytest.raises(ps.PsError) as e:
        ps.ps_predict_load(model, ids, offs, None, pf, pt, ps.alloc_workspace(256, dev))
    assert e.value.code == -5
    assert ps.ps_workspace_bytes(model, -1, 4) == 0
    info = model.info
    assert (info.layers, info.hidden, info.heads, info.ffn, info.vocab, info.dtype) == (2, 128, 2, 512, 8192, 0)
