"""Pins for the CPU oracle of the load-look-ahead map in KV-token units (paper Sec. 3.4.1): hand
cases, closed forms, the section's rule iterated on fractions, round trips, skipped records."""
import os

import numpy as np
import pytest

from oracle import lookahead as ol

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "lookahead_hand_cases.txt")


def read_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if not t:
            continue
        if t[0] == "case":
            cur = {"name": t[1], "n_inst": int(t[2]), "map_len": int(t[3]), "recs": [], "rows": {}, "ovf": {}}
            cases.append(cur)
        elif t[0] == "rec":
            cur["recs"].append([int(v) for v in t[1:]])
        elif t[0] == "row":
            cur["rows"][int(t[1])] = [int(v) for v in t[2:]]
        elif t[0] == "overflow":
            cur["ovf"][int(t[1])] = int(t[2])
    return cases


def run(recs, n_inst, map_len, **kw):
    a = np.array(recs, np.int32).reshape(-1, 6)
    return ol.lookahead_update(a[:, 0], a[:, 1], a[:, 2], a[:, 3], a[:, 4], a[:, 5], n_inst, map_len, **kw)


@pytest.mark.parametrize("case", read_cases(), ids=lambda c: c["name"])
def test_hand_cases(case):
    kv, ovf, st, bad = run(case["recs"], case["n_inst"], case["map_len"])
    want = np.zeros((case["n_inst"], case["map_len"]), np.int32)
    for k, row in case["rows"].items():
        want[k] = row
    want_ovf = np.zeros(case["n_inst"], np.int64)
    for k, v in case["ovf"].items():
        want_ovf[k] = v
    assert st == 0 and bad == -1
    assert np.array_equal(kv, want) and np.array_equal(ovf, want_ovf)


@pytest.mark.parametrize("P,D,s", [(0, 1, 0), (7, 1, 5), (100, 50, 3), (911, 632, 0), (4096, 4096, 0), (1, 300, 3796)])
def test_admit_values_and_closed_form_sum(P, D, s):
    """A request holds P + i tokens at its i-th iteration; the sum over the map is D P + D (D - 1) / 2."""
    L = 4096
    kv, ovf, st, _ = run([[0, s, P, 0, D, 1]], 1, L)
    inside = min(D, L - s)
    assert st == 0
    assert np.array_equal(kv[0, s:s + inside], P + np.arange(inside))
    assert kv[0, :s].sum() == 0 and kv[0, s + inside:].sum() == 0
    assert int(kv.sum()) + int(ovf[0]) == D * P + D * (D - 1) // 2
    # what falls beyond the map: iterations L - s .. D - 1
    i = np.arange(inside, D, dtype=np.int64)
    assert int(ovf[0]) == int((P + i).sum())


def test_matches_the_printed_rule_on_fractions():
    """U'_i = (U_i M + (P + i)) / M iterated request by request in floating point gives N / M."""
    rng = np.random.default_rng(3)
    L, M = 600, 163840.0
    recs, U = [], np.zeros(L)
    for _ in range(200):
        s, P, D = int(rng.integers(0, L)), int(rng.integers(1, 900)), int(rng.integers(1, 700))
        recs.append([0, s, P, 0, D, 1])
        U = ol.paper_rule_on_fractions(U, M, s, P, D)
        if rng.random() < 0.3:                           # finished early after D' iterations
            d_hat = int(rng.integers(0, D))
            recs.append([0, s, P, d_hat, D, -1])
            U = ol.paper_rule_on_fractions(U, M, s, P, D, sign=-1, i_begin=d_hat)
    kv, _, st, _ = run(recs, 1, L)
    assert st == 0
    np.testing.assert_allclose(ol.fraction(kv, [M])[0], U, rtol=0, atol=1e-12)


def test_add_then_subtract_is_identity_and_order_free():
    rng = np.random.default_rng(4)
    n, K, L = 500, 7, 300
    recs = np.stack([rng.integers(0, K, n), rng.integers(0, L, n), rng.integers(0, 2000, n),
                     np.zeros(n, np.int64), rng.integers(0, 400, n), np.ones(n, np.int64)], 1)
    base = rng.integers(-50, 50, (K, L)).astype(np.int32)
    kv, ovf, st, _ = run(recs, K, L, kv_tokens=base)
    assert st == 0 and not np.array_equal(kv, base)
    back = recs.copy()
    back[:, 5] = -1
    kv2, ovf2, st2, _ = run(back[rng.permutation(n)], K, L, kv_tokens=kv, overflow=ovf)
    assert st2 == 0 and np.array_equal(kv2, base) and not ovf2.any()
    # any order of the same records gives the same map
    kv3, ovf3, _, _ = run(recs[rng.permutation(n)], K, L, kv_tokens=base)
    assert np.array_equal(kv3, kv) and np.array_equal(ovf3, ovf)


def test_split_ranges_compose():
    """[0, D) equals [0, c) then [c, D): an extension is the continuation of the same ramp."""
    whole = run([[2, 10, 33, 0, 90, 1]], 4, 128)
    parts = run([[2, 10, 33, 0, 40, 1], [2, 10, 33, 40, 90, 1]], 4, 128)
    assert np.array_equal(whole[0], parts[0]) and np.array_equal(whole[1], parts[1])


def test_bad_records_are_skipped_and_reported():
    good = [0, 1, 5, 0, 3, 1]
    bad = [[3, 1, 5, 0, 3, 1], [-1, 1, 5, 0, 3, 1], [0, 8, 5, 0, 3, 1], [0, -1, 5, 0, 3, 1], [0, 1, -5, 0, 3, 1],
           [0, 1, 1 << 20, 0, 3, 1], [0, 1, 5, -1, 3, 1], [0, 1, 5, 4, 3, 1], [0, 1, 5, 0, 65536, 1],
           [0, 1, 5, 0, 3, 0], [0, 1, 5, 0, 3, 2]]
    want = run([good], 3, 8)[0]
    for i, b in enumerate(bad):
        kv, ovf, st, first = run([good, b, good], 3, 8)
        assert st == 1 and first == 1, (i, b)
        assert np.array_equal(kv, 2 * want)
    kv, _, st, first = run([[0, 1, 5, 2, 2, 1]], 3, 8)            # empty range: valid, no effect
    assert st == 0 and first == -1 and not kv.any()


def test_int32_range_is_reported():
    kv, _, st, _ = run([[0, 0, 1000, 0, 2, 1]], 1, 4, kv_tokens=np.full((1, 4), 2**31 - 1001, np.int32))
    assert st == 2
    assert kv[0, 0] == 2**31 - 1 and kv[0, 1] == np.int32(-2**31)    # second slot wrapped: low 32 bits
