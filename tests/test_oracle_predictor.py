"""Pins for the predictor oracle: properties the mathematics fixes, brute force on 1-3 token
prompts, closed forms, hand-worked values and PyTorch's own fp64 encoder as an independent
library routine.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import predictor as op
from paper_2504_03702_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "head_and_rounding_cases.txt")
TINY = wl.MODELS["tiny"]


def tiny_model(tmp_models, name="tiny.bin", cfg=TINY, weights=None, **kw):
    path = os.path.join(tmp_models, name)
    w = weights if weights is not None else wl.make_weights(cfg, seed=0, **kw)
    wl.write_model(path, cfg, w)
    return op.load_model(path), w


# ------------------------------------------------------------------ softmax / LayerNorm
def test_softmax_rows_sum_to_one_and_uniform():
    rng = np.random.default_rng(0)
    s = rng.normal(0, 30, (50, 37))
    w = op.softmax_rows(s)
    assert np.all(np.abs(w.sum(axis=1) - 1) < 1e-12) and np.all(w >= 0)
    assert np.allclose(op.softmax_rows(np.full((3, 8), 5.0)), 1 / 8, atol=0, rtol=1e-15)
    assert np.allclose(op.softmax_rows(s + 1000.0), w, rtol=1e-9)          # shift invariance
    row = op.softmax_rows(np.array([[0.0, math.log(3.0)]]))
    assert np.allclose(row, [[0.25, 0.75]], rtol=1e-14)


def test_layer_norm_properties():
    rng = np.random.default_rng(1)
    v = rng.normal(3, 2, (7, 64))
    one, zero = np.ones(64), np.zeros(64)
    y = op.layer_norm(v, one, zero, 1e-12)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-13)
    var = v.var(axis=1)                                  # biased
    assert np.allclose(y.var(axis=1), var / (var + 1e-12), rtol=1e-12)
    g, b = rng.normal(1, 0.1, 64), rng.normal(0, 0.1, 64)
    assert np.allclose(op.layer_norm(v, g, b, 1e-12), y * g + b, rtol=1e-12)
    assert np.array_equal(op.layer_norm(np.full((2, 64), 4.2), g, b, 1e-12), np.tile(b, (2, 1)))
    # a two-element row (1, 3): mean 2, biased variance 1 -> (-1, 1)
    assert np.allclose(op.layer_norm(np.array([[1.0, 3.0]]), np.ones(2), np.zeros(2), 0.0), [[-1, 1]])


def test_gelu_values():
    z = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    phi = np.array([0.5 * (1 + math.erf(t / math.sqrt(2))) for t in z])
    assert np.allclose(op.gelu(z), z * phi, rtol=1e-15)
    assert op.gelu(np.array([0.0]))[0] == 0.0
    assert abs(op.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15     # Phi(1)


# ------------------------------------------------------------------ attention by brute force
def brute_force_attention(x, lay, heads):
    """Triple loops with math.exp; written without looking at the oracle's own function."""
    S, H = x.shape
    d = H // heads
    def lin(row, W, b):
        return [sum(row[i] * W[i][j] for i in range(H)) + b[j] for j in range(H)]
    q = [lin(x[p], lay["W_q"], lay["b_q"]) for p in range(S)]
    k = [lin(x[p], lay["W_k"], lay["b_k"]) for p in range(S)]
    v = [lin(x[p], lay["W_v"], lay["b_v"]) for p in range(S)]
    out = np.zeros((S, H))
    for a in range(heads):
        for p in range(S):
            sc = [sum(q[p][a * d + i] * k[t][a * d + i] for i in range(d)) / math.sqrt(d) for t in range(S)]
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            for i in range(d):
                out[p, a * d + i] = sum(e[t] / z * v[t][a * d + i] for t in range(S))
    return out


@pytest.mark.parametrize("S", [1, 2, 3])
def test_attention_brute_force_short_prompts(S):
    rng = np.random.default_rng(10 + S)
    H, heads = 8, 2
    lay = {n: rng.normal(0, 0.7, (H, H)) for n in ("W_q", "W_k", "W_v")}
    lay.update({n: rng.normal(0, 0.3, H) for n in ("b_q", "b_k", "b_v")})
    x = rng.normal(0, 1, (S, H))
    got = op.self_attention(x, lay, heads)
    assert np.allclose(got, brute_force_attention(x, lay, heads), rtol=1e-12, atol=1e-13)
    if S == 1:      # a single token attends to itself with weight 1: output is its value row
        assert np.allclose(got[0], x[0] @ lay["W_v"] + lay["b_v"], rtol=1e-14)


# ------------------------------------------------------------------ PyTorch fp64 as a library check
def torch_layer_from(lay, H, heads, F, eps):
    m = torch.nn.TransformerEncoderLayer(H, heads, F, dropout=0.0, activation="gelu",
                                         layer_norm_eps=eps, batch_first=True, norm_first=False,
                                         dtype=torch.float64)
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    with torch.no_grad():
        m.self_attn.in_proj_weight.copy_(t(np.concatenate([lay["W_q"].T, lay["W_k"].T, lay["W_v"].T])))
        m.self_attn.in_proj_bias.copy_(t(np.concatenate([lay["b_q"], lay["b_k"], lay["b_v"]])))
        m.self_attn.out_proj.weight.copy_(t(lay["W_o"].T)); m.self_attn.out_proj.bias.copy_(t(lay["b_o"]))
        m.linear1.weight.copy_(t(lay["W_1"].T)); m.linear1.bias.copy_(t(lay["b_1"]))
        m.linear2.weight.copy_(t(lay["W_2"].T)); m.linear2.bias.copy_(t(lay["b_2"]))
        m.norm1.weight.copy_(t(lay["ln_1"][0])); m.norm1.bias.copy_(t(lay["ln_1"][1]))
        m.norm2.weight.copy_(t(lay["ln_2"][0])); m.norm2.bias.copy_(t(lay["ln_2"][1]))
    return m.eval()


def test_encoder_layer_equals_torch_fp64(tmp_models):
    model, _ = tiny_model(tmp_models, "tiny_jit.bin", ln_jitter=0.1, bias_std=0.05)
    lay = model["layer"][1]
    x = np.random.default_rng(2).normal(0, 1, (19, TINY.hidden))
    ref = torch_layer_from(lay, TINY.hidden, TINY.heads, TINY.ffn, 1e-12)
    with torch.no_grad():
        want = ref(torch.tensor(x).unsqueeze(0))[0].numpy()
    got = op.encoder_layer(x, lay, TINY.heads, 1e-12)
    assert np.abs(got - want).max() < 1e-10


def test_whole_predictor_equals_torch_composition(tmp_models):
    """Embedding + positions + embedding LayerNorm + stacked layers + [CLS] + head, built from
    torch modules in fp64 on a padded batch with a key-padding mask."""
    model, _ = tiny_model(tmp_models, "tiny_jit.bin", ln_jitter=0.1, bias_std=0.05)
    H = TINY.hidden
    rng = np.random.default_rng(4)
    lengths = np.array([5, 1, 17, 9], np.int32)
    ids = rng.integers(0, TINY.vocab, int(lengths.sum())).astype(np.int32)
    batch = wl.pad_prompts(lengths, ids)
    smax = int(lengths.max())
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    tok = torch.tensor(batch.token_ids.reshape(4, smax).astype(np.int64))
    e = t(model["E_tok"])[tok] + t(model["E_pos"])[:smax].unsqueeze(0)
    x = torch.nn.functional.layer_norm(e, (H,), t(model["ln_e"][0]), t(model["ln_e"][1]), 1e-12)
    mask = torch.arange(smax).unsqueeze(0) >= torch.tensor(lengths.astype(np.int64)).unsqueeze(1)
    with torch.no_grad():
        for lay in model["layer"]:
            x = torch_layer_from(lay, H, TINY.heads, TINY.ffn, 1e-12)(x, src_key_padding_mask=mask)
        c = x[:, 0, :]
        y = torch.relu(c @ t(model["W_h1"]) + t(model["b_h1"])) @ t(model["w_h2"]) + t(model["b_h2"])
    pred_f, pred_tok = op.predict_load(model, batch.token_ids, batch.offsets, batch.lengths)
    assert np.abs(pred_f - y.numpy()).max() < 1e-8
    assert np.array_equal(pred_tok, np.clip(np.rint(y.numpy()), 0, 4096).astype(np.int32))
    assert np.ptp(pred_f) > 1.0            # the four prompts do get different predictions


# ------------------------------------------------------------------ closed forms, invariances
def test_zero_weights_closed_form(tmp_models):
    cfg = TINY
    w = {k: np.zeros_like(v) for k, v in wl.make_weights(cfg, 0).items()}
    rng = np.random.default_rng(6)
    H = cfg.hidden
    w["layer1.ln_2.beta"] = rng.normal(0, 1, H).astype(np.float32)
    w["W_h1"] = rng.normal(0, 0.1, (H, H)).astype(np.float32)
    w["b_h1"] = rng.normal(0, 0.1, H).astype(np.float32)
    w["w_h2"] = rng.normal(0, 1, H).astype(np.float32)
    w["b_h2"] = np.array([7.0], np.float32)
    model, _ = tiny_model(tmp_models, "tiny_zero.bin", weights=w)
    b = wl.make_prompts("tiny", 1)
    pred_f, _ = op.predict_load(model, b.token_ids, b.offsets)
    # every LayerNorm sees a constant row (all gammas are 0), so the final state is ln_2.beta
    beta = w["layer1.ln_2.beta"].astype(np.float64)
    h = np.maximum(beta @ w["W_h1"].astype(np.float64) + w["b_h1"], 0)
    want = h @ w["w_h2"].astype(np.float64) + 7.0
    assert np.allclose(pred_f, want, rtol=1e-13)


def test_batch_order_and_padding_invariance(tmp_models):
    model, _ = tiny_model(tmp_models)
    b = wl.make_prompts("tiny", 2, n_req=6)
    lengths = b.valid_lengths()
    base, base_tok = op.predict_load(model, b.token_ids, b.offsets)
    perm = np.array([3, 0, 5, 1, 4, 2])
    chunks = [b.token_ids[b.offsets[r]:b.offsets[r + 1]] for r in range(6)]
    pb = wl.pack_prompts(lengths[perm], np.concatenate([chunks[r] for r in perm]))
    p, _ = op.predict_load(model, pb.token_ids, pb.offsets)
    assert np.array_equal(p, base[perm])
    padded = wl.pad_prompts(lengths, b.token_ids, pad_id=123)
    q, q_tok = op.predict_load(model, padded.token_ids, padded.offsets, padded.lengths)
    assert np.array_equal(q, base) and np.array_equal(q_tok, base_tok)
    # a request alone gives what it gives inside a batch
    solo, _ = op.predict_load(model, chunks[4], np.array([0, len(chunks[4])]))
    assert solo[0] == base[4]


def test_soft_prompts_are_appended_tokens(tmp_models):
    """With E_soft[j] = E_tok[u_j], (text, M learnable prompts) must equal (text ++ u, M = 0)."""
    import dataclasses
    cfg_soft = dataclasses.replace(TINY, n_soft=4)
    w = wl.make_weights(TINY, 0, ln_jitter=0.05, bias_std=0.02)
    u = np.array([11, 4097, 8191, 0])
    ws = dict(w)
    ws["E_soft"] = w["E_tok"][u].copy()
    plain, _ = tiny_model(tmp_models, "tiny_plain.bin", cfg=TINY, weights=w)
    soft, _ = tiny_model(tmp_models, "tiny_soft.bin", cfg=cfg_soft, weights=ws)
    b = wl.make_prompts("tiny", 3, n_req=5)
    lengths = b.valid_lengths()
    ext_ids = np.concatenate([np.concatenate([b.token_ids[b.offsets[r]:b.offsets[r + 1]], u]) for r in range(5)])
    ext = wl.pack_prompts(lengths + 4, ext_ids)
    a, _ = op.predict_load(soft, b.token_ids, b.offsets)
    c, _ = op.predict_load(plain, ext.token_ids, ext.offsets)
    assert np.array_equal(a, c)
    base, _ = op.predict_load(plain, b.token_ids, b.offsets)
    assert np.abs(a - base).max() > 1e-6          # and the prompts do change the prediction


def test_position_embeddings_matter(tmp_models):
    model, _ = tiny_model(tmp_models)
    ids = np.array([5, 9, 9, 700], np.int32)
    a, _ = op.predict_load(model, ids, np.array([0, 4]))
    b, _ = op.predict_load(model, ids[[0, 3, 2, 1]], np.array([0, 4]))
    assert abs(a[0] - b[0]) > 1e-9


# ------------------------------------------------------------------ hand-worked values
def golden_lines(kind):
    with open(GOLDEN) as f:
        return [l.split()[1:] for l in f if l.startswith(kind + " ")]


def test_head_hand_example():
    (want,), = golden_lines("head")
    model = dict(W_h1=np.array([[1.0, 2.0], [3.0, -1.0]]), b_h1=np.array([0.5, -1.0]),
                 w_h2=np.array([2.0, -3.0]), b_h2=np.array([10.0]))
    assert op.regression_head(model, np.array([1.0, -2.0])) == float(want)


def test_rounding_table():
    rows = golden_lines("round")
    vals = np.array([float(v) for v, _ in rows])
    assert op.to_tokens(vals, 4096).tolist() == [int(t) for _, t in rows]
    with pytest.raises(op.OracleError):
        op.to_tokens(np.array([1.0, float("nan")]), 4096)


def test_errors(tmp_models):
    model, _ = tiny_model(tmp_models)
    with pytest.raises(op.OracleError):
        op.predict_load(model, np.array([1, 8192]), np.array([0, 2]))
    with pytest.raises(op.OracleError):
        op.predict_load(model, np.array([1, 2]), np.array([0, 0, 2]))
    with pytest.raises(op.OracleError):
        op.predict_load(model, np.zeros(200, np.int32), np.array([0, 200]))


def test_bf16_file_is_widened_exactly(tmp_models):
    import dataclasses
    cfg = dataclasses.replace(TINY, dtype=wl.DTYPE_BF16)
    w = wl.make_weights(cfg, 0)
    path = os.path.join(tmp_models, "tiny_bf16.bin")
    wl.write_model(path, cfg, w)
    m = op.load_model(path)
    assert np.array_equal(m["E_tok"], w["E_tok"].astype(np.float64))
    assert np.array_equal(m["layer"][1]["W_2"], w["layer1.W_2"].astype(np.float64))
    assert np.array_equal(m["w_h2"], w["w_h2"].astype(np.float64))
    bits = wl.fp32_to_bf16_bits(np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -0.1], np.float32))
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 1.5*2^-8 rounds up; 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert bits.tolist()[:4] == [0x3F80, 0x3F80, 0x3F81, 0x3F82]
