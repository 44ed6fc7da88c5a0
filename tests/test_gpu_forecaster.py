"""GPU parity of ps_forecast (service workload predictor's online phase, paper Sec. 3.2, Alg. 2)
against the fp64 oracle on the same seeded models and histories, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import forecaster as of
from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-4          # fp32 recurrence of k + 1 steps against fp64


def run_forecast(x):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)
    S = x.hist_p.shape[0]
    out = torch.full((S * 5,), -1.0, dtype=torch.float32, device=DEV)
    ps.ps_forecast(t(x.weights).reshape(-1), x.hidden, t(x.hist_p).reshape(-1), t(x.hist_d).reshape(-1), S, x.k,
                   t(x.mu).reshape(-1), out)
    return out.cpu().numpy().reshape(S, 5).T.astype(np.float64)


@pytest.mark.parametrize("S,H,k", [(1, 1, 1), (3, 8, 4), (8, 32, 12), (5, 64, 24), (130, 17, 9)])
def test_forecasts_and_instance_counts(S, H, k):
    print(f"forecast S={S} H={H} k={k}", flush=True)
    x = wl.make_forecaster_inputs(seed=S + H, n_services=S, hidden=H, k=k)
    got = run_forecast(x)
    ref = of.forecast_services([x.model(s, 0) for s in range(S)], [x.model(s, 1) for s in range(S)],
                               x.hist_p.astype(np.float64), x.hist_d.astype(np.float64),
                               x.mu[:, 0].astype(np.float64), x.mu[:, 1].astype(np.float64), x.mu[:, 2].astype(np.float64))
    scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref ** 2, axis=1, keepdims=True)))
    err = np.abs(got - ref) / scale
    print(f"  max rel err {err.max():.2e}", flush=True)
    assert err.max() < TOL
    assert np.std(ref[2]) > 0 or S == 1                      # services differ
    if S >= 8:
        # both kinds of second step occur: first forecast inside the history's range (recurrence carried on) and
        # outside it (extended history normalised afresh)
        inside = (ref[0] >= x.hist_p.min(axis=1)) & (ref[0] <= x.hist_p.max(axis=1))
        assert inside.any() and (~inside).any()


def test_argument_checks():
    z = torch.zeros(16, dtype=torch.float32, device=DEV)
    with pytest.raises(ps.PsError) as e:
        load = ps.load_library()
        ps._check(load.ps_forecast(z.data_ptr(), 65, z.data_ptr(), z.data_ptr(), 1, 1, z.data_ptr(), z.data_ptr(), None),
                  "ps_forecast")
    assert e.value.code == -6
