"""Pins for the oracle's fixed-iteration form of Algorithm 2 (the paper's implementation runs 10 halvings)."""
import numpy as np

import oracle


def _numpy_bisect(row, p, iters):
    """Separately written loop over Algorithm 2's inner steps (numpy, fp64)."""
    a = row.astype(np.float64)
    target = float(np.float32(p)) * a.sum()
    lo, hi = 0.0, a.max()
    for _ in range(iters):
        mid = (hi + lo) / 2
        if a[a >= mid].sum() < target:
            hi = mid
        else:
            lo = mid
    return np.nonzero(a >= lo)[0], lo


def test_hand_worked_rows():
    # p = 0.7, max = 0.5: mid 0.25 keeps 0.75 >= 0.7 -> low = 0.25; every later midpoint in (0.25, 0.5]
    # keeps only 0.5 < 0.7 -> high comes down, low stays: the set is {0, 1} after any number of steps
    row = np.array([[0.5, 0.25, 0.125, 0.125]], dtype=np.float32)
    for k in (1, 2, 10):
        res = oracle.bisection_select(row, 0.7, k)
        assert list(res.row_set(0)) == [0, 1] and res.tau[0] == np.float32(0.25)
    # an attention sink: 10 halvings of [0, 0.9] cannot reach thresholds below 0.9 / 1024, the tail needed
    # for p = 0.95 lies below that, so low never leaves 0 and every position is kept - zeros included
    x = 0.1 / (3 * 2047)
    sink = np.zeros((1, 4096), dtype=np.float32)
    sink[0, 0] = 0.9
    sink[0, 2:2049], sink[0, 2049:] = 2 * x, x          # position 1 stays exactly zero
    res = oracle.bisection_select(sink, 0.95, 10)
    assert res.counts[0] == 4096 and res.tau[0] == 0.0
    # the exact nucleus: the sink and the 2047 heavier tail entries (0.9 + 0.0667 >= 0.95)
    exact = oracle.topp_select(sink, 0.95)
    assert exact.counts[0] == 2048 and list(exact.row_set(0)[:3]) == [0, 2, 3]


def test_agrees_with_separate_numpy_loop():
    rng = np.random.default_rng(0)
    probs = rng.dirichlet(np.full(700, 0.2), size=8).astype(np.float32)
    for k in (3, 10, 25):
        res = oracle.bisection_select(probs, 0.9, k)
        for r in range(8):
            if res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
                continue
            want, lo = _numpy_bisect(probs[r], 0.9, k)
            assert np.array_equal(res.row_set(r), want)
            assert float(res.tau[r]) >= lo and (res.tau[r] == 0 or float(np.nextafter(res.tau[r], np.float32(0))) < lo)


def test_contains_the_exact_nucleus_and_converges_to_it():
    rng = np.random.default_rng(1)
    probs = rng.dirichlet(np.full(512, 0.3), size=6).astype(np.float32)
    lens = np.array([512, 300, 1, 17, 512, 64], dtype=np.int32)
    for r in range(6):
        probs[r, lens[r]:] = 0.0
    exact = oracle.topp_select(probs, 0.9, lens)
    prev = None
    for k in (2, 6, 10, 60):
        res = oracle.bisection_select(probs, 0.9, k, lens)
        for r in range(6):
            assert set(exact.row_set(r)) <= set(res.row_set(r))             # theta_low <= tau*: a superset
            assert (res.row_set(r) < lens[r]).all()
            if prev is not None:
                assert set(res.row_set(r)) <= set(prev.row_set(r))          # more halvings never add positions
        prev = res
    for r in range(6):
        if not (exact.flags[r] | prev.flags[r]) & oracle.ROW_NEAR_BOUNDARY:
            assert np.array_equal(prev.row_set(r), exact.row_set(r))        # 60 halvings: the same set


def test_invalid_rows():
    probs = np.full((3, 8), 0.125, dtype=np.float32)
    probs[0, 3] = np.nan
    probs[1] = 0.0
    res = oracle.bisection_select(probs, 0.9, 10)
    assert res.flags[0] & oracle.ROW_INVALID and res.flags[1] & oracle.ROW_INVALID and res.counts[:2].sum() == 0
    assert res.counts[2] == 8
