"""Pins for the CPU oracle of the router's scoring (paper Sec. 3.4.3)."""
import numpy as np

from oracle import router as orr


def test_no_memory_pressure_is_join_shortest_queue_with_low_index_ties():
    """With empty maps far from T_mem the score is queued prefill + decode tokens + the request."""
    K, l = 3, 8
    win = np.zeros((K, l), np.int64)
    a, s, win2, qp, cd = orr.route([10, 10, 10, 10], [5, 5, 5, 5], win, [10**6] * K, [0, 0, 0], [0, 0, 0])
    assert a.tolist() == [0, 1, 2, 0]                     # ties go to the lowest index, then round robin
    assert s.tolist() == [1500, 1500, 1500, 3000]
    assert qp.tolist() == [20, 10, 10] and cd.tolist() == [10, 5, 5]
    assert win2[0].tolist() == [20, 22, 24, 26, 28, 0, 0, 0]   # two requests: 2 * (10 + t) for t < 5


def test_memory_penalty_moves_a_request_away_from_a_full_instance():
    # instance 0 is idle in queue terms but its map peaks at 900 of 1000 tokens; instance 1 has a queue
    win = np.array([[900] * 4, [0] * 4])
    # P = 50, D = 4: on instance 0 the peak becomes 900 + 53 = 953 -> penalty 100*953 - 80*1000 = 15300
    a, s, *_ = orr.route([50], [4], win, [1000, 1000], [0, 100], [0, 0])
    assert a.tolist() == [1] and s.tolist() == [100 * (100 + 50 + 0 + 4)]
    # with a longer queue on instance 1 the penalised instance wins: 100 * 54 + 15300 = 20700
    a, s, *_ = orr.route([50], [4], win, [1000, 1000], [0, 200], [0, 0])
    assert a.tolist() == [0] and s.tolist() == [20700]


def test_the_ramp_only_counts_inside_the_window_and_while_decoding():
    win = np.array([[0, 0, 0, 700, 0, 0]])
    # D = 2: iterations 0, 1 hold 100, 101; the peak stays the 700 already in the map (below T_mem)
    _, s, win2, *_ = orr.route([100], [2], win, [1000], [0], [0])
    assert s.tolist() == [100 * 102] and win2[0].tolist() == [100, 101, 0, 700, 0, 0]
    # D = 10 > l: the ramp covers the whole window; the peak is 700 + 103 = 803 -> penalty 300
    _, s, win2, *_ = orr.route([100], [10], win, [1000], [0], [0])
    assert s.tolist() == [100 * 110 + 300] and win2[0].tolist() == [100, 101, 102, 803, 104, 105]


def test_later_requests_see_earlier_decisions():
    K, l = 2, 4
    win = np.zeros((K, l), np.int64)
    # capacities so small that the first request's ramp makes instance 0 pay the penalty next time
    a, s, *_ = orr.route([40, 40, 40], [4, 4, 4], win, [50, 50], [0, 0], [0, 0])
    # r0 -> 0 (tie). r1: instance 0 has queue 44 and peak 2*43; instance 1 is empty -> 1. r2: symmetric again -> 0
    assert a.tolist() == [0, 1, 0]
    assert s[0] == 100 * 44 + (100 * 43 - 80 * 50)


def test_requests_without_a_prediction_are_not_dispatched():
    win = np.zeros((2, 4), np.int64)
    a, s, win2, qp, cd = orr.route([10, 10, -3], [5, -1, 5], win, [1000, 1000], [0, 0], [0, 0])
    assert a.tolist() == [0, -1, -1] and s.tolist() == [1500, 0, 0]
    assert qp.tolist() == [10, 0] and cd.tolist() == [5, 0]
