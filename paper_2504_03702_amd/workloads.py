"""Seeded synthetic inputs for the request-load-predictor + load-anticipator path.

This module only draws random numbers and lays them out in files and arrays.  It
holds none of the method's arithmetic (no encoder, no head, no anticipator) and is
imported by the tests and the benchmark to feed both the GPU library and the CPU
oracle with the same bytes.  It imports neither of them.

Shapes follow the paper's workload description (Sec. 2.2 "Challenge 2": prompt
lengths 7..911 tokens, median 52; responses 5..632, median 87; Sec. 3.4.1: response
lengths up to 4096).  Prompt contents and traces themselves are not available, so
token ids, lengths, arrivals and instance assignments are drawn from the stated
distributions with ``numpy.random.default_rng(seed)`` in a fixed order.

Model file layout (little endian), read independently by the GPU library and by the
oracle:

    bytes 0..7    magic  b"PSLP0001"
    bytes 8..47   int32  layers, hidden, heads, ffn, vocab, max_pos, n_soft,
                         head_hidden, dtype (0 = fp32, 1 = bf16), d_max
    bytes 48..55  float64 LayerNorm epsilon
    bytes 56..63  zero padding
    then the tensors below, back to back, each row-major in the file's dtype.
    Linear maps are stored [in][out]:  y = x @ W + b.

      E_tok [vocab, hidden]   E_pos [max_pos, hidden]   E_soft [n_soft, hidden]
      ln_e.gamma [hidden]     ln_e.beta [hidden]
      per layer:  W_q [H,H] b_q [H]  W_k [H,H] b_k [H]  W_v [H,H] b_v [H]
                  W_o [H,H] b_o [H]  ln_1.gamma [H] ln_1.beta [H]
                  W_1 [H,F] b_1 [F]  W_2 [F,H] b_2 [H]  ln_2.gamma [H] ln_2.beta [H]
      head:       W_h1 [H,Hh]  b_h1 [Hh]  w_h2 [Hh]  b_h2 [1]
"""
from __future__ import annotations

import dataclasses
import struct
from typing import Dict, List, Optional, Tuple

import numpy as np

MAGIC = b"PSLP0001"
HEADER_BYTES = 64
DTYPE_FP32 = 0
DTYPE_BF16 = 1


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    layers: int
    hidden: int
    heads: int
    ffn: int
    vocab: int
    max_pos: int
    n_soft: int = 0
    head_hidden: int = 0          # 0 -> same as hidden
    dtype: int = DTYPE_BF16
    d_max: int = 4096             # longest response the paper considers (Sec. 3.4.1, Table 2)
    ln_eps: float = 1e-12

    def resolved(self) -> "ModelConfig":
        if self.head_hidden == 0:
            return dataclasses.replace(self, head_hidden=self.hidden)
        return self


# The encoder shapes of the five benchmark configurations.
MODELS: Dict[str, ModelConfig] = {
    "tiny": ModelConfig(2, 128, 2, 512, 8192, 128, dtype=DTYPE_FP32),
    "bert_base": ModelConfig(12, 768, 12, 3072, 30522, 512),
    "latency": ModelConfig(6, 768, 12, 3072, 30522, 512),          # DistilBERT's own shape
    "production": ModelConfig(16, 1024, 16, 4096, 30522, 2048),
}


def tensor_specs(cfg: ModelConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the tensors in file order."""
    cfg = cfg.resolved()
    H, F, Hh = cfg.hidden, cfg.ffn, cfg.head_hidden
    specs: List[Tuple[str, Tuple[int, ...]]] = [
        ("E_tok", (cfg.vocab, H)),
        ("E_pos", (cfg.max_pos, H)),
        ("E_soft", (cfg.n_soft, H)),
        ("ln_e.gamma", (H,)),
        ("ln_e.beta", (H,)),
    ]
    for l in range(cfg.layers):
        p = f"layer{l}."
        specs += [
            (p + "W_q", (H, H)), (p + "b_q", (H,)),
            (p + "W_k", (H, H)), (p + "b_k", (H,)),
            (p + "W_v", (H, H)), (p + "b_v", (H,)),
            (p + "W_o", (H, H)), (p + "b_o", (H,)),
            (p + "ln_1.gamma", (H,)), (p + "ln_1.beta", (H,)),
            (p + "W_1", (H, F)), (p + "b_1", (F,)),
            (p + "W_2", (F, H)), (p + "b_2", (H,)),
            (p + "ln_2.gamma", (H,)), (p + "ln_2.beta", (H,)),
        ]
    specs += [("W_h1", (H, Hh)), ("b_h1", (Hh,)), ("w_h2", (Hh,)), ("b_h2", (1,))]
    return specs


# --------------------------------------------------------------------------- bf16 storage
def fp32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store_round(x: np.ndarray, dtype: int) -> np.ndarray:
    """Value as it will read back from the file (fp32 array, exactly representable)."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == DTYPE_BF16:
        return bf16_bits_to_fp32(fp32_to_bf16_bits(x)).reshape(x.shape)
    return x


# --------------------------------------------------------------------------- weights
def make_weights(cfg: ModelConfig, seed: int = 0, *, ln_jitter: float = 0.0,
                 bias_std: float = 0.0, head_bias: float = 128.0,
                 head_scale: float = 800.0) -> Dict[str, np.ndarray]:
    """Random-init weights: matrices and embeddings N(0, 0.02), LayerNorm gamma 1 / beta 0,
    biases 0.  The regression head's output layer is scaled (w_h2 ~ head_scale * N(0, 0.02),
    b_h2 = head_bias) so that untrained predictions spread over a few hundred tokens rather
    than all rounding to zero.  ``ln_jitter`` / ``bias_std`` > 0 perturb gammas, betas and
    biases so parity tests exercise those terms too.  Values are returned as fp32 arrays
    already rounded to the file's storage dtype."""
    cfg = cfg.resolved()
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape in tensor_specs(cfg):
        base = name.split(".")[-1]
        n = int(np.prod(shape)) if len(shape) else 1
        if base == "gamma":
            v = np.ones(shape, np.float32)
            if ln_jitter:
                v = v + ln_jitter * rng.standard_normal(shape, dtype=np.float32)
        elif base == "beta":
            v = np.zeros(shape, np.float32)
            if ln_jitter:
                v = v + ln_jitter * rng.standard_normal(shape, dtype=np.float32)
        elif name == "b_h2":
            v = np.full(shape, head_bias, np.float32)
        elif base.startswith("b_"):
            v = np.zeros(shape, np.float32)
            if bias_std:
                v = v + bias_std * rng.standard_normal(shape, dtype=np.float32)
        elif name == "w_h2":
            v = (0.02 * head_scale) * rng.standard_normal(shape, dtype=np.float32)
        else:
            v = 0.02 * rng.standard_normal(shape, dtype=np.float32) if n else np.zeros(shape, np.float32)
        out[name] = _store_round(v, cfg.dtype)
    return out


def write_model(path: str, cfg: ModelConfig, weights: Dict[str, np.ndarray]) -> None:
    cfg = cfg.resolved()
    with open(path, "wb") as f:
        hdr = MAGIC + struct.pack(
            "<10i", cfg.layers, cfg.hidden, cfg.heads, cfg.ffn, cfg.vocab, cfg.max_pos,
            cfg.n_soft, cfg.head_hidden, cfg.dtype, cfg.d_max) + struct.pack("<d", cfg.ln_eps)
        f.write(hdr.ljust(HEADER_BYTES, b"\0"))
        for name, shape in tensor_specs(cfg):
            w = np.asarray(weights[name], dtype=np.float32).reshape(shape)
            if cfg.dtype == DTYPE_BF16:
                f.write(fp32_to_bf16_bits(w).tobytes())
            else:
                f.write(w.astype("<f4").tobytes())


# --------------------------------------------------------------------------- prompts
def lognormal_lengths(rng: np.random.Generator, n: int, mu: float, sigma: float,
                      lo: int, hi: int) -> np.ndarray:
    return np.clip(np.rint(np.exp(rng.normal(mu, sigma, n))), lo, hi).astype(np.int32)


def zipf_ids(rng: np.random.Generator, n: int, vocab: int, s: float = 1.1) -> np.ndarray:
    """ids with P(id = k-1) proportional to k^-s, k = 1..vocab (bounded Zipf, inverse CDF)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    return np.minimum(np.searchsorted(cdf, rng.random(n), side="left"), vocab - 1).astype(np.int32)


@dataclasses.dataclass
class PromptBatch:
    token_ids: np.ndarray            # int32, packed or padded
    offsets: np.ndarray              # int32 [n_req + 1]
    lengths: Optional[np.ndarray]    # int32 [n_req] valid lengths (padded layout) or None (packed)

    @property
    def n_req(self) -> int:
        return int(self.offsets.shape[0] - 1)

    def valid_lengths(self) -> np.ndarray:
        if self.lengths is not None:
            return self.lengths
        return np.diff(self.offsets).astype(np.int32)


def pack_prompts(lengths: np.ndarray, ids: np.ndarray) -> PromptBatch:
    offsets = np.zeros(len(lengths) + 1, np.int32)
    offsets[1:] = np.cumsum(lengths)
    return PromptBatch(ids.astype(np.int32), offsets, None)


def pad_prompts(lengths: np.ndarray, ids: np.ndarray, pad_id: int = 0) -> PromptBatch:
    """Same prompts as ``pack_prompts`` laid out padded to the batch maximum."""
    n, smax = len(lengths), int(lengths.max())
    padded = np.full((n, smax), pad_id, np.int32)
    start = 0
    for r, s in enumerate(lengths):
        padded[r, :s] = ids[start:start + s]
        start += int(s)
    offsets = (np.arange(n + 1, dtype=np.int64) * smax).astype(np.int32)
    return PromptBatch(padded.reshape(-1), offsets, lengths.astype(np.int32))


def make_prompts(kind: str, seed: int = 0, n_req: Optional[int] = None) -> PromptBatch:
    """Prompt batches of the five configurations.  ``n_req`` overrides the batch size."""
    rng = np.random.default_rng(seed + 1000)
    if kind == "tiny":
        n = n_req or 16
        lengths = rng.integers(8, 65, n).astype(np.int32)
        ids = rng.integers(0, MODELS["tiny"].vocab, int(lengths.sum())).astype(np.int32)
        return pack_prompts(lengths, ids)
    if kind == "bert_base_padded":
        n = n_req or 64
        lengths = lognormal_lengths(rng, n, 5.3, 0.8, 4, 512)
        ids = rng.integers(0, 30522, int(lengths.sum())).astype(np.int32)
        return pad_prompts(lengths, ids)
    if kind == "bert_base_varlen":
        n = n_req or 1024
        lengths = lognormal_lengths(rng, n, 5.3, 1.0, 4, 512)
        ids = zipf_ids(rng, int(lengths.sum()), 30522, 1.1)
        return pack_prompts(lengths, ids)
    if kind == "latency":
        n = n_req or 8
        lengths = lognormal_lengths(rng, n, 5.0, 0.9, 4, 512)
        ids = rng.integers(0, 30522, int(lengths.sum())).astype(np.int32)
        return pack_prompts(lengths, ids)
    if kind == "production":
        n = n_req or 4096
        lengths = lognormal_lengths(rng, n, 5.5, 1.2, 4, 2048)
        ids = rng.integers(0, 30522, int(lengths.sum())).astype(np.int32)
        return pack_prompts(lengths, ids)
    raise ValueError(kind)


def poisson_arrival_times(seed: int, n: int, rate_per_s: float) -> np.ndarray:
    """Arrival times (seconds) of a Poisson stream: cumulative exponential gaps."""
    rng = np.random.default_rng(seed + 2000)
    return np.cumsum(rng.exponential(1.0 / rate_per_s, n))


# --------------------------------------------------------------------------- anticipator
@dataclasses.dataclass
class AnticipatorInputs:
    pred_tokens: np.ndarray          # int32 [n]
    instance_id: np.ndarray          # int32 [n]
    arrival_bucket: np.ndarray       # int32 [n]
    rate: Optional[np.ndarray]       # int32 [n_inst] tokens/s per instance, or None
    n_inst: int
    horizon: int


def make_anticipator_inputs(kind: str, seed: int = 0, n: Optional[int] = None,
                            pred_tokens: Optional[np.ndarray] = None) -> AnticipatorInputs:
    """Instance assignment, arrival buckets and decode rates.  ``pred_tokens`` may be given
    (the predictor's output); otherwise response lengths are drawn from a lognormal matched
    to the paper's response-length median 87 and P5..P95 = 5..632, clipped to [1, 4096]."""
    rng = np.random.default_rng(seed + 3000)
    if kind == "tiny":
        n_inst, horizon, with_rate, n = 4, 64, False, n or 16
    elif kind == "small":
        n_inst, horizon, with_rate, n = 4, 64, True, n or 64
    elif kind == "medium":
        n_inst, horizon, with_rate, n = 64, 600, True, n or 1024
    elif kind in ("production", "stream", "stream_by_arrival"):
        n_inst, horizon, with_rate = 256, 600, True
        n = n or (4096 if kind == "production" else 44_100_000)
    else:
        raise ValueError(kind)
    instance = rng.integers(0, n_inst, n, dtype=np.int32)
    arrival = rng.integers(0, horizon, n, dtype=np.int32)
    if kind == "stream_by_arrival":
        arrival.sort()                      # a request log: records in the order the requests arrive
    rate = rng.integers(30, 61, n_inst, dtype=np.int32) if with_rate else None
    if pred_tokens is None:
        pred_tokens = np.clip(np.rint(np.exp(rng.normal(np.log(87.0), 1.3, n))), 1, 4096).astype(np.int32)
    else:
        pred_tokens = np.asarray(pred_tokens, np.int32)
        assert pred_tokens.shape[0] == n
    return AnticipatorInputs(pred_tokens, instance, arrival, rate, n_inst, horizon)


@dataclasses.dataclass
class LookaheadInputs:
    """Records of the look-ahead map in KV-token units (paper Sec. 3.4.1): one row per column."""
    instance_id: np.ndarray
    start_iter: np.ndarray
    prompt_tokens: np.ndarray
    i_begin: np.ndarray
    i_end: np.ndarray
    sign: np.ndarray
    capacity: np.ndarray          # [n_inst] token capacity M of each instance
    n_inst: int
    map_len: int

    def columns(self):
        return (self.instance_id, self.start_iter, self.prompt_tokens, self.i_begin, self.i_end, self.sign)


def make_lookahead_inputs(kind: str, seed: int = 0, n: Optional[int] = None,
                          pred_tokens: Optional[np.ndarray] = None,
                          prompt_tokens: Optional[np.ndarray] = None) -> LookaheadInputs:
    """A stream of map updates: every request is admitted (ramp over [0, D)); a share of them also
    carries its correction, as the paper describes them: finished early after D' < D iterations (the
    rest subtracted), or still running at D (a virtual extension of ceil(0.2 D) iterations added, its
    unused part subtracted when the request completes inside it).  Prompt lengths follow the prompt
    statistics (lognormal, median 52, clipped to [7, 2048]) unless given, response lengths the
    response statistics unless given; the map has one slot per decoding iteration up to the model's
    maximum output (4096); start slots are uniform over the first quarter of the map."""
    rng = np.random.default_rng(seed + 5000)
    if kind == "tiny":
        n_inst, map_len, n = 3, 64, n or 24
    elif kind == "medium":
        n_inst, map_len, n = 64, 1024, n or 2048
    elif kind in ("production", "stream"):
        n_inst, map_len = 256, 4096
        n = n or (4096 if kind == "production" else 10_000_000)
    else:
        raise ValueError(kind)
    if pred_tokens is None:
        d = np.clip(np.rint(np.exp(rng.normal(np.log(87.0), 1.3, n))), 1, 4096).astype(np.int64)
    else:
        d = np.clip(np.asarray(pred_tokens, np.int64), 0, 4096)
    if prompt_tokens is None:
        p = np.clip(np.rint(np.exp(rng.normal(np.log(52.0), 1.2, n))), 7, 2048).astype(np.int64)
    else:
        p = np.asarray(prompt_tokens, np.int64)
    if kind == "tiny":
        d, p = np.minimum(d, 40), np.minimum(p, 30)
    k = rng.integers(0, n_inst, n)
    s = rng.integers(0, max(map_len // 4, 1), n)
    fate = rng.random(n)
    early = fate < 0.3
    late = (fate >= 0.3) & (fate < 0.5)
    d_hat = np.where(early, (rng.random(n) * d).astype(np.int64), d)           # D' in [0, D)
    ext = np.ceil(0.2 * d).astype(np.int64)
    used = np.where(late, np.minimum(ext, (rng.random(n) * (ext + 1)).astype(np.int64)), 0)
    cols = [np.stack([k, s, p, np.zeros(n, np.int64), d, np.ones(n, np.int64)], 1),
            np.stack([k, s, p, d_hat, d, -np.ones(n, np.int64)], 1)[early],
            np.stack([k, s, p, d, d + ext, np.ones(n, np.int64)], 1)[late],
            np.stack([k, s, p, d + used, d + ext, -np.ones(n, np.int64)], 1)[late]]
    rec = np.concatenate(cols, 0)
    rec = rec[rng.permutation(rec.shape[0])].astype(np.int32)
    capacity = rng.integers(120_000, 400_001, n_inst).astype(np.int32)
    return LookaheadInputs(*[np.ascontiguousarray(rec[:, c]) for c in range(6)], capacity, n_inst, map_len)



FORECASTER_FIELDS = ("w_mx", "W_mh", "w_hx", "W_hm", "b_h", "w_ix", "W_im", "b_i", "w_ox", "W_om", "b_o", "w_fx", "W_fm",
                     "b_f", "w_out", "b_out")


@dataclasses.dataclass
class ForecasterInputs:
    """Models and histories of the service workload predictor (paper Sec. 3.2)."""
    weights: np.ndarray           # [n_services, 2, 5 H^2 + 10 H + 1] float32, fields in FORECASTER_FIELDS order
    hist_p: np.ndarray            # [n_services, k] float32 prompt tokens per past window
    hist_d: np.ndarray            # [n_services, k] float32 response tokens per past window
    mu: np.ndarray                # [n_services, 3] float32 per-instance capacities (prefill, decode, total)
    hidden: int
    k: int

    def model(self, s: int, kind: int) -> dict:
        """Model `kind` (0 prompt, 1 response) of service s as named float64 arrays."""
        H, flat, at, out = self.hidden, self.weights[s, kind].astype(np.float64), 0, {}
        for n in FORECASTER_FIELDS:
            size = H * H if n.startswith("W_") else 1 if n == "b_out" else H
            v = flat[at:at + size]
            # matrices are stored input-major ([in][out]); the named arrays are [out][in]
            out[n] = v.reshape(H, H).T.copy() if n.startswith("W_") else v[0] if n == "b_out" else v
            at += size
        return out


def make_forecaster_inputs(seed: int = 0, n_services: int = 8, hidden: int = 32, k: int = 12) -> ForecasterInputs:
    """Random-init models (N(0, 0.3) matrices, N(0, 0.5) vectors, read-out weights N(0, 0.5) and bias 0.5, so that
    first forecasts fall inside the history's range for some services and outside it for others) and histories
    shaped like the paper's traces: token counts per 10-minute window following a daily cycle with noise, prompt
    tokens around 4e6 and response tokens around 2e6 per window."""
    rng = np.random.default_rng(seed + 7000)
    H = hidden
    per_model = 5 * H * H + 10 * H + 1
    w = np.zeros((n_services, 2, per_model), np.float32)
    for s in range(n_services):
        for kind in range(2):
            parts = []
            for n in FORECASTER_FIELDS:
                if n.startswith("W_"):
                    parts.append(rng.normal(0, 0.3, H * H))
                elif n == "b_out":
                    parts.append(np.array([0.5]))
                else:
                    parts.append(rng.normal(0, 0.5, H))
            w[s, kind] = np.concatenate(parts).astype(np.float32)
    t = np.arange(k)[None, :] + rng.integers(0, 144, (n_services, 1))
    cycle = 1.0 + 0.5 * np.sin(2 * np.pi * t / 144.0)
    hist_p = (4e6 * cycle * rng.uniform(0.8, 1.2, (n_services, k))).astype(np.float32)
    hist_d = (2e6 * cycle * rng.uniform(0.8, 1.2, (n_services, k))).astype(np.float32)
    mu = np.stack([rng.uniform(0.8e6, 1.6e6, n_services), rng.uniform(0.3e6, 0.8e6, n_services),
                   rng.uniform(1.0e6, 2.0e6, n_services)], 1).astype(np.float32)
    return ForecasterInputs(w, hist_p, hist_d, mu, hidden, k)

