"""CPU oracle for the online phase of the service workload predictor (paper Sec. 3.2, Alg. 2): a
multiplicative LSTM per service and token kind forecasts the token count of the next time window from
the counts of the previous k windows, in two steps, and the counts are turned into a number of
instances.

TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.  It shares no
code with the GPU path; only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

A model sees its input sequence min-max normalised (Alg. 1's normalisation step, the form the models
are trained on):  x_t = (v_t - min v) / (max v - min v)  over the sequence it is given, and its
output is taken back to token counts with the same two numbers:  forecast = min v + (max v - min v) y,
not below 0.  A flat sequence (max v = min v) takes the range as 1.

The recurrence is the multiplicative LSTM of Krause et al. (2016), which the paper names: with scalar
input x_t, hidden state h and cell c,
    m_t = (w_mx x_t) * (W_mh h_{t-1})                      elementwise product
    hh  = w_hx x_t + W_hm m_t + b_h
    i_t = sigmoid(w_ix x_t + W_im m_t + b_i),  o_t, f_t likewise
    c_t = f_t * c_{t-1} + i_t * tanh(hh)
    h_t = tanh(c_t) * o_t
and the model's output after the last input is  y = w_out . h + b_out.
Online phase (Alg. 2): step 1 applies the model to the k past windows and gives the forecast of the
current window; that forecast is appended to the history and step 2 applies the model to the k + 1
values (normalised over those k + 1 values) for the next window.  With both kinds forecast, prompt
tokens P and response tokens D,
    N = max(P / mu_p, D / mu_d, (P + D) / mu_t)
for the instance's profiled prefill, decode and total token capacities per window."""
from __future__ import annotations

import numpy as np

NAMES = ("w_mx", "W_mh", "w_hx", "W_hm", "b_h", "w_ix", "W_im", "b_i", "w_ox", "W_om", "b_o", "w_fx", "W_fm", "b_f",
         "w_out", "b_out")


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def mlstm_step(w, x, h, c):
    m = (w["w_mx"] * x) * (w["W_mh"] @ h)
    hh = w["w_hx"] * x + w["W_hm"] @ m + w["b_h"]
    i = sigmoid(w["w_ix"] * x + w["W_im"] @ m + w["b_i"])
    o = sigmoid(w["w_ox"] * x + w["W_om"] @ m + w["b_o"])
    f = sigmoid(w["w_fx"] * x + w["W_fm"] @ m + w["b_f"])
    c = f * c + i * np.tanh(hh)
    return np.tanh(c) * o, c


def normalise(seq):
    """Alg. 1's normalisation of one input sequence: (normalised values, minimum, range)."""
    seq = np.asarray(seq, np.float64)
    lo, hi = float(seq.min()), float(seq.max())
    span = hi - lo if hi > lo else 1.0
    return (seq - lo) / span, lo, span


def model_forecast(w, seq):
    """The model applied to one sequence of token counts: normalise, run the recurrence, read out, de-normalise."""
    w = {k: np.asarray(v, np.float64) for k, v in w.items()}
    x, lo, span = normalise(seq)
    hm = w["W_mh"].shape[0]
    h, c = np.zeros(hm), np.zeros(hm)
    for xt in x:
        h, c = mlstm_step(w, xt, h, c)
    y = float(w["w_out"] @ h) + float(w["b_out"])
    return max(0.0, lo + span * y)


def two_step_forecast(w, history):
    """(forecast of the current window, forecast of the next window) from the k past windows."""
    history = np.asarray(history, np.float64)
    y1 = model_forecast(w, history)
    return y1, model_forecast(w, np.append(history, y1))


def forecast_services(models_p, models_d, hist_p, hist_d, mu_p, mu_d, mu_t):
    """Per service s: (P_cur, D_cur, P_next, D_next, N_next) as float64 arrays."""
    S = len(models_p)
    out = np.zeros((5, S))
    for s in range(S):
        p1, p2 = two_step_forecast(models_p[s], hist_p[s])
        d1, d2 = two_step_forecast(models_d[s], hist_d[s])
        out[:, s] = (p1, d1, p2, d2, max(p2 / mu_p[s], d2 / mu_d[s], (p2 + d2) / mu_t[s]))
    return out
