"""CPU oracle for the request load predictor (paper Sec. 3.3 "Tier-2: Request Load
Prediction"): prompt token ids -> predicted response length.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain fp64 definition the GPU library is
checked against.  It shares no code with the GPU path and must never be used by it;
only tests, the smoke check and the benchmark's CPU-baseline leg call it.

What the paper fixes (Sec. 3.3): the encoder is DistilBERT, a distilled BERT; the final
hidden state of the first token ([CLS]) is the sequence representation; a two-layer
feed-forward network maps it to the length prediction; M learnable prompt vectors are
appended to the input text tokens.  Everything the paper leaves to "DistilBERT" follows
the published DistilBERT / BERT encoder: learned absolute positions, embedding LayerNorm,
post-LayerNorm residual blocks, scaled dot-product attention over the request's own
tokens (bidirectional), erf-GELU feed-forward, biases on every linear map.

Each request is processed on its own, one step after the other, with no blocking or
fusion; numpy's matmul and scipy's erf serve as library primitives.
"""
from __future__ import annotations

import struct
from typing import Dict, Optional, Tuple

import numpy as np
from scipy.special import erf

_MAGIC = b"PSLP0001"


class OracleError(ValueError):
    def __init__(self, what: str, index: int = -1):
        super().__init__(f"{what} (index {index})")
        self.what = what
        self.index = index


# ----------------------------------------------------------------------------- model file
def _read_tensor(buf: memoryview, pos: int, shape, dtype: int) -> Tuple[np.ndarray, int]:
    n = int(np.prod(shape))
    if dtype == 1:      # bf16: the high half of an fp32, widened exactly
        bits = np.frombuffer(buf, dtype="<u2", count=n, offset=pos)
        val = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        pos += 2 * n
    else:
        val = np.frombuffer(buf, dtype="<f4", count=n, offset=pos).astype(np.float64)
        pos += 4 * n
    return val.reshape(shape), pos


def load_model(path: str) -> Dict[str, object]:
    """Read a model file into fp64 arrays (stored values widened exactly, never re-rounded)."""
    with open(path, "rb") as f:
        raw = f.read()
    if len(raw) < 64 or raw[:8] != _MAGIC:
        raise OracleError("bad model file header")
    L, H, A, F, V, P, M, Hh, dt, dmax = struct.unpack_from("<10i", raw, 8)
    (eps,) = struct.unpack_from("<d", raw, 48)
    if min(L, H, A, F, V, P, Hh) < 1 or M < 0 or dt not in (0, 1) or H % A:
        raise OracleError("bad model file header")
    m: Dict[str, object] = dict(layers=L, hidden=H, heads=A, ffn=F, vocab=V, max_pos=P,
                                n_soft=M, head_hidden=Hh, dtype=dt, d_max=dmax, ln_eps=eps)
    buf, pos = memoryview(raw), 64

    def take(shape):
        nonlocal pos
        t, pos = _read_tensor(buf, pos, shape, dt)
        return t

    m["E_tok"], m["E_pos"], m["E_soft"] = take((V, H)), take((P, H)), take((M, H))
    m["ln_e"] = (take((H,)), take((H,)))
    layers = []
    for _ in range(L):
        lay = {}
        for k in ("q", "k", "v", "o"):
            lay["W_" + k], lay["b_" + k] = take((H, H)), take((H,))
            if k == "o":
                lay["ln_1"] = (take((H,)), take((H,)))
        lay["W_1"], lay["b_1"] = take((H, F)), take((F,))
        lay["W_2"], lay["b_2"] = take((F, H)), take((H,))
        lay["ln_2"] = (take((H,)), take((H,)))
        layers.append(lay)
    m["layer"] = layers
    m["W_h1"], m["b_h1"], m["w_h2"], m["b_h2"] = take((H, Hh)), take((Hh,)), take((Hh,)), take((1,))
    if pos != len(raw):
        raise OracleError("model file size does not match its header")
    return m


# ----------------------------------------------------------------------------- the steps
def layer_norm(v: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """LayerNorm over the last axis with the biased variance."""
    mean = v.mean(axis=-1, keepdims=True)
    var = ((v - mean) ** 2).mean(axis=-1, keepdims=True)
    return gamma * (v - mean) / np.sqrt(var + eps) + beta


def softmax_rows(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def gelu(z: np.ndarray) -> np.ndarray:
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def embed(model, ids: np.ndarray) -> np.ndarray:
    """Rows of one request: its text tokens, then the M learnable prompt vectors (Sec. 3.3:
    they are appended to the input text tokens), each plus the position embedding of its
    index within the request, then the embedding LayerNorm."""
    n, M = len(ids), model["n_soft"]
    e = np.concatenate([model["E_tok"][ids], model["E_soft"]], axis=0) + model["E_pos"][: n + M]
    return layer_norm(e, *model["ln_e"], model["ln_eps"])


def self_attention(x: np.ndarray, lay, heads: int) -> np.ndarray:
    """Multi-head scaled dot-product attention of one request over its own S rows."""
    S, H = x.shape
    d = H // heads
    q = x @ lay["W_q"] + lay["b_q"]
    k = x @ lay["W_k"] + lay["b_k"]
    v = x @ lay["W_v"] + lay["b_v"]
    o = np.empty_like(x)
    for a in range(heads):
        sl = slice(a * d, (a + 1) * d)
        w = softmax_rows(q[:, sl] @ k[:, sl].T / np.sqrt(d))
        o[:, sl] = w @ v[:, sl]
    return o


def encoder_layer(x: np.ndarray, lay, heads: int, eps: float) -> np.ndarray:
    o = self_attention(x, lay, heads)
    x1 = layer_norm(x + o @ lay["W_o"] + lay["b_o"], *lay["ln_1"], eps)
    g = gelu(x1 @ lay["W_1"] + lay["b_1"])
    return layer_norm(x1 + g @ lay["W_2"] + lay["b_2"], *lay["ln_2"], eps)


def regression_head(model, c: np.ndarray) -> float:
    """Two-layer feed-forward network on the [CLS] state (Sec. 3.3)."""
    h = np.maximum(c @ model["W_h1"] + model["b_h1"], 0.0)
    return float(h @ model["w_h2"] + model["b_h2"][0])


def to_tokens(y: np.ndarray, d_max: int) -> np.ndarray:
    """Round half to even, then clamp to [0, d_max] (responses are at most d_max tokens)."""
    y = np.asarray(y, dtype=np.float64)
    if np.isnan(y).any():
        raise OracleError("prediction is NaN", int(np.flatnonzero(np.isnan(y))[0]))
    return np.clip(np.rint(y), 0, d_max).astype(np.int32)


def encode_request(model, ids: np.ndarray) -> np.ndarray:
    """Final hidden states [S, H] of one request."""
    x = embed(model, ids)
    for lay in model["layer"]:
        x = encoder_layer(x, lay, model["heads"], model["ln_eps"])
    return x


def predict_load(model, token_ids: np.ndarray, offsets: np.ndarray,
                 lengths: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """pred_f[r] (fp64) and pred_tokens[r] (int32) for every request.

    Request r's text tokens are token_ids[offsets[r] : offsets[r] + S_r] with
    S_r = lengths[r] if ``lengths`` is given (the rest of the span is padding and takes no
    part in anything) else offsets[r+1] - offsets[r].  The caller puts [CLS] first."""
    token_ids = np.asarray(token_ids)
    offsets = np.asarray(offsets, dtype=np.int64)
    n_req = len(offsets) - 1
    pred = np.empty(n_req, dtype=np.float64)
    for r in range(n_req):
        span = int(offsets[r + 1] - offsets[r])
        s = int(lengths[r]) if lengths is not None else span
        if s < 1 or s > span:
            raise OracleError("request length out of range", r)
        if s + model["n_soft"] > model["max_pos"]:
            raise OracleError("request longer than the position table", r)
        ids = token_ids[offsets[r]: offsets[r] + s].astype(np.int64)
        if ids.min() < 0 or ids.max() >= model["vocab"]:
            raise OracleError("token id out of range", r)
        x = encode_request(model, ids)
        pred[r] = regression_head(model, x[0])
    return pred, to_tokens(pred, model["d_max"])
