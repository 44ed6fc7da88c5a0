"""CPU oracle for the load-aware request router's scoring (paper Sec. 3.4.3) over a micro-batch of
requests, written out plainly.

TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.  It shares no
code with the GPU path; only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

For a request with P prompt tokens and D predicted response tokens the estimated load of instance i is
    L_i = (queued_p_i + P) + (current_d_i + D) + beta * max(0, U_i - T_mem) * M_i
where U_i is the peak, over the next l iterations, of instance i's look-ahead map with the request
virtually added (P + t tokens at iteration t < D, Sec. 3.4.1), M_i its token capacity and T_mem the
usage that incurs no preemption (80 %).  The request goes to the instance with the smallest L_i (the
lowest index on ties); that instance's queued prefill tokens, decode tokens and look-ahead window are
then updated, so the next request of the micro-batch sees the decision.  Everything is kept in token
units and whole percents (T_mem as an integer percent), so scores are integers:
    100 L_i = 100 (queued_p_i + P + current_d_i + D) + beta * max(0, 100 peak_i - T_pct M_i)."""
from __future__ import annotations

import numpy as np


def route(prompt_tokens, pred_tokens, window_tokens, capacity, queued_p, current_d, t_mem_pct: int = 80,
          beta: int = 1):
    """window_tokens [K, l] int: the next l iterations of every instance's map (copied, then updated).
    Returns (assigned [n] int32, score100 [n] int64 of the chosen instance, window, queued_p, current_d)."""
    win = np.array(window_tokens, np.int64)
    K, l = win.shape
    qp = np.array(queued_p, np.int64)
    cd = np.array(current_d, np.int64)
    M = np.asarray(capacity, np.int64)
    n = len(prompt_tokens)
    assigned = np.zeros(n, np.int32)
    score = np.zeros(n, np.int64)
    for r in range(n):
        P, D = int(prompt_tokens[r]), int(pred_tokens[r])
        if P < 0 or D < 0:                      # no such request (e.g. a failed prediction): not dispatched
            assigned[r], score[r] = -1, 0
            continue
        best, best_i = None, -1
        for i in range(K):
            peak = -2**62
            for t in range(l):
                v = int(win[i, t]) + (P + t if t < D else 0)
                peak = max(peak, v)
            pen = max(0, 100 * peak - t_mem_pct * int(M[i])) if l > 0 else 0
            L = 100 * (int(qp[i]) + P + int(cd[i]) + D) + beta * pen
            if best is None or L < best:
                best, best_i = L, i
        assigned[r], score[r] = best_i, best
        qp[best_i] += P
        cd[best_i] += D
        for t in range(min(D, l)):
            win[best_i, t] += P + t
    return assigned, score, win, qp, cd
