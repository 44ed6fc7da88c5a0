"""Pins for the anticipator oracle: hand-worked cases, the totals invariant, a second
formulation (difference array + prefix sum, written independently here), order independence,
accumulation and error reporting.  CPU only."""
import os

import numpy as np
import pytest

from oracle import anticipator as oa
from paper_2504_03702_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "anticipator_hand_cases.txt")


def hand_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, mid, tail = [p.split() for p in line.split("|")]
            hz, rate, a, d = map(int, head)
            cases.append((hz, rate, a, d, list(map(int, mid)), int(tail[0])))
    return cases


@pytest.mark.parametrize("hz,rate,a,d,expect,ovf", hand_cases())
def test_hand_cases(hz, rate, a, d, expect, ovf):
    r = None if rate < 0 else [rate]
    load, overflow, st, bad = oa.anticipate([d], [0], [a], r, 1, hz)
    assert st == 0 and bad == -1
    assert load[0].tolist() == expect
    assert int(overflow[0]) == ovf


def by_difference_array(inp):
    """Independent formulation: a request is two range-adds, [a, a+rem) gets q+1 and
    [a+rem, a+dur) gets q; range-adds become point updates of a difference array whose
    prefix sum is the curve.  Extended past the horizon so the tail sums to the overflow."""
    K, Hz = inp.n_inst, inp.horizon
    ext = Hz + int(inp.pred_tokens.max()) + 2
    diff = np.zeros((K, ext + 1), np.int64)
    for D, k, a in zip(inp.pred_tokens.tolist(), inp.instance_id.tolist(), inp.arrival_bucket.tolist()):
        if D == 0:
            continue
        dur = Hz - a if inp.rate is None else -(-D // int(inp.rate[k]))
        q, rem = divmod(D, dur)
        diff[k, a] += q + 1
        diff[k, a + rem] -= 1
        diff[k, a + dur] -= q
    curve = np.cumsum(diff, axis=1)
    return curve[:, :Hz], curve[:, Hz:].sum(axis=1)


@pytest.mark.parametrize("kind,n", [("tiny", 16), ("small", 64), ("medium", 1024), ("production", 4096)])
def test_matches_difference_array_and_totals(kind, n):
    inp = wl.make_anticipator_inputs(kind, seed=3, n=n)
    load, overflow, st, _ = oa.anticipate(inp.pred_tokens, inp.instance_id, inp.arrival_bucket,
                                          inp.rate, inp.n_inst, inp.horizon)
    assert st == 0
    ref_load, ref_ovf = by_difference_array(inp)
    assert np.array_equal(load, ref_load)
    assert np.array_equal(overflow, ref_ovf)
    # totals: every instance's curve plus overflow holds exactly its requests' predicted tokens
    per_inst = np.bincount(inp.instance_id, weights=inp.pred_tokens, minlength=inp.n_inst).astype(np.int64)
    assert np.array_equal(load.sum(axis=1, dtype=np.int64) + overflow, per_inst)
    if inp.rate is None:
        assert not overflow.any()


def test_no_bucket_exceeds_rate_per_request():
    # with a decode rate, a single request never puts more than rate tokens in a bucket
    for D in range(1, 400):
        for rate in (1, 7, 30, 60):
            load, ovf, _, _ = oa.anticipate([D], [0], [0], [rate], 1, 512)
            assert load.max() <= rate and load.sum() + ovf.sum() == D
            dur = -(-D // rate)
            assert np.count_nonzero(load) == min(dur, 512)
            assert load[0, 0] - load[0, dur - 1] in (0, 1)      # as even as integers allow


def test_order_independence_and_accumulation():
    inp = wl.make_anticipator_inputs("medium", seed=5, n=2000)
    full = oa.anticipate(inp.pred_tokens, inp.instance_id, inp.arrival_bucket, inp.rate, inp.n_inst, inp.horizon)
    perm = np.random.default_rng(0).permutation(2000)
    shuf = oa.anticipate(inp.pred_tokens[perm], inp.instance_id[perm], inp.arrival_bucket[perm],
                         inp.rate, inp.n_inst, inp.horizon)
    assert np.array_equal(full[0], shuf[0]) and np.array_equal(full[1], shuf[1])
    # two calls that accumulate equal one call over the concatenation
    h = 900
    first = oa.anticipate(inp.pred_tokens[:h], inp.instance_id[:h], inp.arrival_bucket[:h], inp.rate,
                          inp.n_inst, inp.horizon)
    second = oa.anticipate(inp.pred_tokens[h:], inp.instance_id[h:], inp.arrival_bucket[h:], inp.rate,
                           inp.n_inst, inp.horizon, load=first[0], overflow=first[1])
    assert np.array_equal(full[0], second[0]) and np.array_equal(full[1], second[1])


def test_bad_records_are_skipped_and_reported():
    pred = [5, -1, 5, 5, 5, 5]
    inst = [0, 0, 2, 0, -1, 1]
    arr = [0, 0, 0, 8, 0, 1]
    load, ovf, st, bad = oa.anticipate(pred, inst, arr, [1, 0], 2, 8)
    assert st == 1 and bad == 1
    assert load[0].tolist() == [1, 1, 1, 1, 1, 0, 0, 0] and not load[1].any() and not ovf.any()


def test_int32_range_is_reported():
    load0 = np.full((1, 4), 2**31 - 2, np.int32)
    load, ovf, st, bad = oa.anticipate([8], [0], [0], None, 1, 4, load=load0)
    assert st == 2 and bad == -1
    assert load[0].tolist() == [-(2**31)] * 4          # low 32 bits of 2^31
