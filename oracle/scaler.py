"""CPU oracle for the in-window checks of the proactive instance scaler (paper Sec. 3.4.2) on the
load-look-ahead maps of Sec. 3.4.1, written out plainly.

TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.  It shares no
code with the GPU path; only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

For each instance, over the next `window` iterations of its map (U = tokens / capacity):
  * it is potentially overloaded if U exceeds `over_pct` % in more than `share_pct` % of those
    iterations (the paper: 95 % in more than 10 %);
  * its peak is max U over the window.
Over all instances: scale-down is allowed if every instance's U stays below `idle_pct` % (the paper's
T_f = 30 %) throughout the window, and the number of instances to isolate is then
N_c - sum_instances(max U) / T_f, with N_c the current instance count.
Percent thresholds are integers so that every comparison is exact: U > p % is tokens * 100 > p * M."""
from __future__ import annotations

import numpy as np


def scaler_scan(kv_tokens, capacity, window: int, over_pct: int = 95, share_pct: int = 10, idle_pct: int = 30):
    """Returns (over_count [K], peak_tokens [K], overloaded [K] 0/1, n_overloaded, all_idle 0/1,
    scale_down float).  Instances with capacity < 1 are skipped (counted neither overloaded nor idle,
    peak 0, contributing nothing to the sum); all_idle is 0 if any is skipped."""
    kv = np.asarray(kv_tokens)
    K, L = kv.shape
    w = min(int(window), L)
    over_count = np.zeros(K, np.int32)
    peak = np.zeros(K, np.int32)
    overloaded = np.zeros(K, np.int32)
    all_idle, total = 1, 0.0
    for k in range(K):
        M = int(capacity[k])
        if M < 1 or w < 1:
            all_idle = 0
            continue
        cnt, pk = 0, -2**31
        for t in range(w):
            n = int(kv[k, t])
            if n * 100 > over_pct * M:
                cnt += 1
            pk = max(pk, n)
        over_count[k], peak[k] = cnt, pk
        overloaded[k] = 1 if cnt * 100 > share_pct * w else 0
        if not pk * 100 < idle_pct * M:
            all_idle = 0
        total += pk / M
    scale_down = K - total / (idle_pct / 100.0)
    return over_count, peak, overloaded, int(overloaded.sum()), all_idle, float(scale_down)
