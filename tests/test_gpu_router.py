"""GPU parity of ps_route (the router's scoring over a micro-batch, paper Sec. 3.4.3) against the
oracle, through the C ABI: decisions, scores and the updated state are integers and must match."""
import numpy as np
import pytest
import torch

from oracle import router as orr
from paper_2504_03702_amd import binding as ps

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_route(P, D, win, cap, qp, cd, **kw):
    K, l = win.shape
    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)
    t64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int64)).to(DEV)
    n = len(P)
    w_t, qp_t, cd_t = t32(win).reshape(-1), t64(qp), t64(cd)
    a_t = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    s_t = torch.full((n,), -7, dtype=torch.int64, device=DEV)
    st = ps.new_status(DEV)
    ps.ps_route(t32(P), t32(D), K, l, w_t if l > 0 else None, t32(cap), qp_t, cd_t, a_t, s_t, status=st, **kw)
    flags, bad = ps.ps_status_read(st)
    return (a_t.cpu().numpy(), s_t.cpu().numpy(), w_t.cpu().numpy().reshape(K, l), qp_t.cpu().numpy(),
            cd_t.cpu().numpy(), flags, bad)


def random_case(rng, K, l, n, hot):
    cap = rng.integers(2000, 6000, K) if hot else rng.integers(100_000, 400_000, K)
    win = rng.integers(0, cap.max() // 2, (K, l))
    qp, cd = rng.integers(0, 3000, K), rng.integers(0, 20000, K)
    P = np.clip(np.rint(np.exp(rng.normal(np.log(52.0), 1.2, n))), 7, 2048).astype(np.int64)
    D = np.clip(np.rint(np.exp(rng.normal(np.log(87.0), 1.3, n))), 0, 4096).astype(np.int64)
    return P, D, win, cap, qp, cd


@pytest.mark.parametrize("K,l,n,hot", [(1, 1, 5, False), (3, 8, 40, True), (4, 100, 300, True), (64, 100, 1000, False),
                                       (256, 100, 4096, True), (256, 100, 512, False), (1000, 30, 200, True),
                                       (17, 333, 100, True), (5, 0, 20, False)])
def test_decisions_scores_and_state_match(K, l, n, hot):
    print(f"route K={K} l={l} n={n} hot={hot}", flush=True)
    P, D, win, cap, qp, cd = random_case(np.random.default_rng(K * 1000 + l), K, l, n, hot)
    a, s, w, q2, c2, flags, _ = run_route(P, D, win, cap, qp, cd)
    ra, rs, rw, rq, rc = orr.route(P, D, win, cap, qp, cd)
    assert flags == 0
    assert np.array_equal(a, ra) and np.array_equal(s, rs)
    assert np.array_equal(w, rw) and np.array_equal(q2, rq) and np.array_equal(c2, rc)
    if K > 1 and n >= 40:
        assert len(np.unique(ra)) > 1                       # the batch really is spread over instances


def test_hand_cases_ties_penalty_and_other_parameters():
    win = np.array([[900] * 4, [0] * 4])
    a, s, *_ = run_route([50], [4], win, [1000, 1000], [0, 200], [0, 0])
    assert a.tolist() == [0] and s.tolist() == [20700]
    a, s, *_ = run_route([50], [4], win, [1000, 1000], [0, 200], [0, 0], beta=2)        # twice the penalty
    assert a.tolist() == [1] and s.tolist() == [100 * 254]
    a, s, *_ = run_route([50], [4], win, [1000, 1000], [0, 200], [0, 0], t_mem_pct=96)   # no penalty yet
    assert a.tolist() == [0] and s.tolist() == [5400]
    a, s, w, qp, cd, *_ = run_route([10] * 4, [5] * 4, np.zeros((3, 8), np.int64), [10**6] * 3, [0] * 3, [0] * 3)
    assert a.tolist() == [0, 1, 2, 0] and qp.tolist() == [20, 10, 10] and w[0].tolist() == [20, 22, 24, 26, 28, 0, 0, 0]


def test_missing_predictions_and_limits():
    win = np.zeros((2, 4), np.int64)
    a, s, w, qp, cd, flags, bad = run_route([10, 10, -3], [5, -1, 5], win, [1000, 1000], [0, 0], [0, 0])
    assert a.tolist() == [0, -1, -1] and s.tolist() == [1500, 0, 0] and qp.tolist() == [10, 0]
    assert flags == ps.PS_ST_BAD_RECORD and bad == 1
    z32 = torch.zeros(2048, dtype=torch.int32, device=DEV)
    z64 = torch.zeros(2048, dtype=torch.int64, device=DEV)
    with pytest.raises(ps.PsError) as e:                    # more instances than one workgroup has threads
        ps.ps_route(z32[:1], z32[:1], 1025, 0, None, z32[:1025], z64[:1025], z64[:1025], z32[:1], z64[:1])
    assert e.value.code == -6
    big = torch.zeros(256 * 200, dtype=torch.int32, device=DEV)
    with pytest.raises(ps.PsError) as e:                    # windows that do not fit the LDS
        ps.ps_route(z32[:1], z32[:1], 256, 200, big, z32[:256], z64[:256], z64[:256], z32[:1], z64[:1])
    assert e.value.code == -6
