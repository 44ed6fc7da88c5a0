"""Pins for the CPU oracle of the scaler's in-window checks (paper Sec. 3.4.2)."""
import numpy as np

from oracle import scaler as osc


def test_overload_needs_more_than_ten_percent_of_the_window_above_95_percent():
    M, l = 1000, 100
    kv = np.zeros((3, 128), np.int32)
    kv[0, :10] = 951          # exactly 10 % of the window above 95 %: not "more than 10 %"
    kv[1, :11] = 951          # 11 %: overloaded
    kv[2, :50] = 950          # exactly 95 % is not above 95 %
    kv[2, 100:] = 999         # beyond the window: ignored
    oc, pk, ov, n_ov, idle, sd = osc.scaler_scan(kv, [M] * 3, l)
    assert oc.tolist() == [10, 11, 0] and ov.tolist() == [0, 1, 0] and n_ov == 1
    assert pk.tolist() == [951, 951, 950] and idle == 0
    # N_c - sum(max U) / T_f
    assert abs(sd - (3 - (0.951 + 0.951 + 0.950) / 0.30)) < 1e-12


def test_scale_down_when_all_stay_below_t_f():
    caps = [1000, 2000, 500, 400]
    kv = np.zeros((4, 64), np.int32)
    kv[0, 5], kv[1, 63], kv[2, 0], kv[3, 7] = 299, 100, 149, 10
    oc, pk, ov, n_ov, idle, sd = osc.scaler_scan(kv, caps, 64)
    assert idle == 1 and n_ov == 0 and not oc.any()
    want = 4 - (0.299 + 0.05 + 0.298 + 0.025) / 0.3
    assert abs(sd - want) < 1e-12
    kv[2, 0] = 150            # exactly 30 % is not below 30 %
    assert osc.scaler_scan(kv, caps, 64)[4] == 0


def test_constant_maps_and_window_clipping():
    kv = np.full((2, 10), 96, np.int32)
    oc, pk, ov, n_ov, idle, _ = osc.scaler_scan(kv, [100, 100], 1000)     # window longer than the map
    assert oc.tolist() == [10, 10] and ov.tolist() == [1, 1] and n_ov == 2 and idle == 0
    oc, pk, ov, *_ = osc.scaler_scan(kv, [100, 0], 4)                     # no capacity: skipped
    assert oc.tolist() == [4, 0] and pk.tolist() == [96, 0] and ov.tolist() == [1, 0]
