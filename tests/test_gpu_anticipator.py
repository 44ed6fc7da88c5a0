"""GPU parity of ps_anticipate against the C oracle: bit-exact histograms on the same seeded
inputs, through the C ABI."""
import dataclasses

import numpy as np
import pytest

from oracle import anticipator as oa
from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
from tests.gpu_util import run_anticipate

pytestmark = pytest.mark.gpu


def check(inp, load0=None, ovf0=None):
    got_load, got_ovf, flags, bad = run_anticipate(inp, load0, ovf0)
    ref_load, ref_ovf, st, ref_bad = oa.anticipate(inp.pred_tokens, inp.instance_id, inp.arrival_bucket, inp.rate,
                                                   inp.n_inst, inp.horizon, load=load0, overflow=ovf0)
    assert np.array_equal(got_load, ref_load)
    assert np.array_equal(got_ovf, ref_ovf)
    assert bool(flags & ps.PS_ST_BAD_RECORD) == bool(st & 1)
    if st & 1:
        assert bad == ref_bad
    return got_load, got_ovf, flags


@pytest.mark.parametrize("kind,n", [("tiny", 16), ("tiny", 1), ("small", 64), ("medium", 1024),
                                    ("production", 4096), ("production", 100_003), ("stream", 3_000_001)])
def test_bit_exact(kind, n):
    print(f"anticipator {kind} n={n}", flush=True)
    inp = wl.make_anticipator_inputs(kind, seed=1, n=n)
    load, ovf, flags = check(inp)
    assert flags == 0
    per_inst = np.bincount(inp.instance_id, weights=inp.pred_tokens, minlength=inp.n_inst).astype(np.int64)
    assert np.array_equal(load.sum(axis=1, dtype=np.int64) + ovf, per_inst)


@pytest.mark.parametrize("n", [262_144, 300_001, 3_000_001])
def test_streams_in_arrival_order(n):
    """Long streams in arrival order take the windowed first kernel (all instances, a window of
    buckets per workgroup); the result is the same bit for bit."""
    print(f"anticipator stream_by_arrival n={n}", flush=True)
    inp = wl.make_anticipator_inputs("stream_by_arrival", seed=4, n=n)
    load, ovf, flags = check(inp)
    assert flags == 0
    per_inst = np.bincount(inp.instance_id, weights=inp.pred_tokens, minlength=inp.n_inst).astype(np.int64)
    assert np.array_equal(load.sum(axis=1, dtype=np.int64) + ovf, per_inst)
    # the same records accumulated a second time into the first result, with an offset overflow
    check(inp, load.copy(), ovf + 7)


def test_arrival_order_with_exceptions():
    """Streams that are almost in arrival order, or whose requests decode for longer than a window, make
    the windowed kernel give up somewhere: the general kernel redoes the call, same result."""
    rng = np.random.default_rng(9)
    base = wl.make_anticipator_inputs("stream_by_arrival", seed=5, n=400_000)
    # a handful of records far from their neighbours' buckets
    a = base.arrival_bucket.copy()
    a[rng.integers(0, a.size, 5)] = rng.integers(0, base.horizon, 5)
    check(dataclasses.replace(base, arrival_bucket=a))
    # slow instances: durations of hundreds of buckets, far beyond a window and the horizon
    check(dataclasses.replace(base, rate=np.full(base.n_inst, 2, np.int32)))
    # invalid records inside an ordered stream are skipped and the first one is named
    k = base.instance_id.copy(); d = base.pred_tokens.copy(); a = base.arrival_bucket.copy()
    k[1234] = base.n_inst; d[200_000] = -3; a[399_999] = base.horizon
    _, _, flags = check(dataclasses.replace(base, instance_id=k, pred_tokens=d, arrival_bucket=a))
    assert flags & ps.PS_ST_BAD_RECORD
    # an invalid (negative) arrival bucket on the very first record, and on the first record of later parts of
    # the stream (400 000 records are folded in 25 parts of 16 000): only those records may be dropped
    for where in ([0], [16_000], [0, 16_000, 32_000, 384_000]):
        print(f"anticipator ordered, negative first bucket at {where}", flush=True)
        a = base.arrival_bucket.copy()
        a[where] = [-2, -1, -7, -600][:len(where)]
        got_load, got_ovf, flags = check(dataclasses.replace(base, arrival_bucket=a))
        assert flags & ps.PS_ST_BAD_RECORD
        keep = np.ones(a.size, bool)
        keep[where] = False
        per_inst = np.bincount(base.instance_id[keep], weights=base.pred_tokens[keep], minlength=base.n_inst).astype(np.int64)
        assert np.array_equal(got_load.sum(axis=1, dtype=np.int64) + got_ovf, per_inst)
    # other shapes: few instances (a window as long as the horizon), many instances (a short window)
    for n_inst, horizon in [(3, 100), (40, 4096), (1200, 600)]:
        print(f"anticipator ordered K={n_inst} Hz={horizon}", flush=True)
        n = 300_000
        inp = wl.AnticipatorInputs(rng.integers(0, 3000, n, dtype=np.int32), rng.integers(0, n_inst, n, dtype=np.int32),
                                   np.sort(rng.integers(0, horizon, n, dtype=np.int32)),
                                   rng.integers(20, 200, n_inst, dtype=np.int32), n_inst, horizon)
        check(inp)


def test_long_streams_in_any_order_with_exceptions():
    """Long streams in no particular order: the windowed kernel sees at once that they are not in arrival order
    and leaves them to the general kernel.  Plain, accumulated, without rates, with large quotients, with the
    largest predictions, with faulty records and a row without a usable rate, and on other shapes."""
    rng = np.random.default_rng(12)
    base = wl.make_anticipator_inputs("stream", seed=6, n=500_000)
    print("anticipator any order: plain", flush=True)
    load, ovf, flags = check(base)
    assert flags == 0
    check(base, load.copy(), ovf + 3)                                  # accumulated a second time
    print("anticipator any order: no rates (spread to the end of the horizon)", flush=True)
    check(dataclasses.replace(base, rate=None))
    print("anticipator any order: fast instances (large quotients)", flush=True)
    check(dataclasses.replace(base, rate=np.full(base.n_inst, 5000, np.int32),
                              pred_tokens=rng.integers(1, 4097, base.pred_tokens.size).astype(np.int32)))
    print("anticipator any order: predictions above 32767", flush=True)
    d = base.pred_tokens.copy()
    d[[7, 250_000, 499_999]] = [40_000, 65_535, 32_768]
    check(dataclasses.replace(base, pred_tokens=d))
    print("anticipator any order: faulty records and a row without a rate", flush=True)
    k = base.instance_id.copy(); d = base.pred_tokens.copy(); a = base.arrival_bucket.copy()
    k[[3, 400_000]] = [-1, base.n_inst]; d[[10, 11]] = [-1, -70_000]; a[[20, 499_000]] = [base.horizon, -5]
    _, _, flags = check(dataclasses.replace(base, instance_id=k, pred_tokens=d, arrival_bucket=a))
    assert flags & ps.PS_ST_BAD_RECORD
    r = base.rate.copy(); r[129] = 0
    check(dataclasses.replace(base, rate=r))
    for n_inst, horizon in [(1200, 600), (129, 1024), (256, 598), (300, 64)]:
        print(f"anticipator any order K={n_inst} Hz={horizon}", flush=True)
        n = 300_000
        inp = wl.AnticipatorInputs(rng.integers(0, 3000, n, dtype=np.int32), rng.integers(0, n_inst, n, dtype=np.int32),
                                   rng.integers(0, horizon, n, dtype=np.int32),
                                   rng.integers(20, 200, n_inst, dtype=np.int32), n_inst, horizon)
        check(inp)


def test_accumulates_into_existing_map():
    inp = wl.make_anticipator_inputs("medium", seed=2, n=5000)
    rng = np.random.default_rng(0)
    load0 = rng.integers(-1000, 1000, (inp.n_inst, inp.horizon)).astype(np.int32)
    ovf0 = rng.integers(0, 10**12, inp.n_inst).astype(np.int64)
    check(inp, load0, ovf0)


def test_odd_shapes_and_many_groups():
    # rows that do not divide into groups evenly, a horizon that is no multiple of anything
    rng = np.random.default_rng(3)
    for n_inst, horizon, n in [(1, 1, 10), (3, 7, 100), (301, 1021, 20000), (37, 9000, 5000), (1000, 64, 30000)]:
        print(f"anticipator odd K={n_inst} Hz={horizon} n={n}", flush=True)
        inp = wl.AnticipatorInputs(rng.integers(0, 5000, n, dtype=np.int32), rng.integers(0, n_inst, n, dtype=np.int32),
                                   rng.integers(0, horizon, n, dtype=np.int32),
                                   rng.integers(1, 200, n_inst, dtype=np.int32), n_inst, horizon)
        check(inp)
        check(dataclasses.replace(inp, rate=None))


def test_divisions_are_exact():
    """The kernel divides by float reciprocals: every (prediction, rate) pair of a dense grid, and
    the extremes of the accepted range, must still give the integer quotients."""
    n_inst = 160
    rates = np.concatenate([np.arange(1, 151), [1 << 19, (1 << 19) - 1, (1 << 19) + 1, 2**31 - 1, 65536, 65537,
                                                 4095, 4096, 4097, 1000]]).astype(np.int32)
    assert rates.shape[0] == n_inst
    D = np.arange(1, 4200, dtype=np.int32)
    pred = np.tile(D, n_inst)
    inst = np.repeat(np.arange(n_inst, dtype=np.int32), D.shape[0])
    arr = (np.arange(pred.shape[0]) % 7).astype(np.int32)
    print("anticipator division grid", flush=True)
    check(wl.AnticipatorInputs(pred, inst, arr, rates, n_inst, 900))
    big = np.array([65535, 65534, 65533, 32768, 32767, 50000, 33333, 9991], np.int32)
    pred = np.tile(big, n_inst)
    inst = np.repeat(np.arange(n_inst, dtype=np.int32), big.shape[0])
    arr = (np.arange(pred.shape[0]) % 900).astype(np.int32)
    check(wl.AnticipatorInputs(pred, inst, arr, rates, n_inst, 900))
    check(wl.AnticipatorInputs(pred, inst, arr, None, n_inst, 900))       # duration = horizon - arrival


def test_bad_records_are_skipped_and_flagged():
    inp = wl.make_anticipator_inputs("small", seed=4, n=500)
    inp.pred_tokens[[17, 400]] = [-5, 65536]
    inp.instance_id[[99, 250]] = [inp.n_inst, -1]
    inp.arrival_bucket[[33, 480]] = [inp.horizon, -2]
    ok = np.ones(500, bool)
    ok[[17, 400, 99, 250, 33, 480]] = False
    got_load, got_ovf, flags, bad = run_anticipate(inp)
    assert flags & ps.PS_ST_BAD_RECORD and bad == 17
    # the oracle has no upper limit on pred_tokens, so compare on the records both accept
    clean = wl.AnticipatorInputs(inp.pred_tokens[ok], inp.instance_id[ok], inp.arrival_bucket[ok], inp.rate,
                                 inp.n_inst, inp.horizon)
    ref_load, ref_ovf, st, _ = oa.anticipate(clean.pred_tokens, clean.instance_id, clean.arrival_bucket, clean.rate,
                                             clean.n_inst, clean.horizon)
    assert st == 0 and np.array_equal(got_load, ref_load) and np.array_equal(got_ovf, ref_ovf)
    bad_rate = dataclasses.replace(clean, rate=np.where(np.arange(inp.n_inst) == 2, 0, inp.rate).astype(np.int32))
    check(bad_rate)


def test_int32_range_is_flagged():
    inp = wl.AnticipatorInputs(np.array([8], np.int32), np.array([0], np.int32), np.array([0], np.int32), None, 1, 4)
    load0 = np.full((1, 4), 2**31 - 2, np.int32)
    got_load, _, flags, _ = run_anticipate(inp, load0)
    assert flags & ps.PS_ST_RANGE
    assert got_load[0].tolist() == [-(2**31)] * 4


def test_host_side_argument_errors():
    import torch
    dev = "cuda:0"
    z = torch.zeros(4, dtype=torch.int32, device=dev)
    load = torch.zeros(8, dtype=torch.int32, device=dev)
    ws = ps.alloc_workspace(ps.ps_anticipate_workspace_bytes(4, 2, 4), dev)
    with pytest.raises(ps.PsError) as e:      # a rate needs an overflow array
        ps.ps_anticipate(z, z, z, torch.ones(2, dtype=torch.int32, device=dev), 2, 4, load, None, ws)
    assert e.value.code == -1
    with pytest.raises(ps.PsError) as e:      # workspace too small
        ps.ps_anticipate(z, z, z, None, 2, 4, load, None, ws[:256].contiguous()[:16])
    assert e.value.code == -5
