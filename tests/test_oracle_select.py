"""Pins for the oracle's top-p selection (CPU only).

Each test fixes the result by something other than the oracle's own code:
hand-worked rows, exhaustive search over subsets (Appendix A, Eq. 8), closed
forms, properties the definition implies, and the paper's own bisection
(Algorithm 2) run until its bracket closes.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2510_27641_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "topp_hand_rows.txt")


def _select1(row, p):
    r = oracle.topp_select(np.asarray(row, dtype=np.float32)[None, :], p)
    return r.row_set(0), float(r.tau[0]), int(r.flags[0])


def test_golden_hand_rows():
    n_cases = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        vals, p, idx, tau = [s.strip() for s in line.split("|")]
        row = [float(x) for x in vals.split()]
        got, got_tau, _ = _select1(row, float(p))
        assert got.tolist() == [int(x) for x in idx.split()], line
        assert got_tau == float(tau), line
        n_cases += 1
    assert n_cases >= 15


def test_boundary_flag_on_exact_hit():
    # 1/2 of the mass is reached exactly by the first entry: on the boundary by construction
    _, _, fl = _select1([0.5, 0.25, 0.125, 0.0625, 0.0625], 0.5)
    assert fl & oracle.ROW_NEAR_BOUNDARY
    _, _, fl = _select1([0.5, 0.25, 0.125, 0.0625, 0.0625], 0.6)
    assert not fl & oracle.ROW_NEAR_BOUNDARY


def test_bruteforce_minimal_subset():
    """Eq. 8 by exhaustive search in exact rational arithmetic, n <= 12, distinct values."""
    rng = np.random.default_rng(11)
    checked = 0
    for trial in range(60):
        n = int(rng.integers(2, 13))
        row = rng.random(n).astype(np.float32) ** 3 + np.float32(1e-3)
        if len(set(row.tolist())) != n:
            continue
        p = float(np.float32(rng.uniform(0.05, 1.0)))
        vals = [Fraction(float(x)) for x in row]
        target = Fraction(p) * sum(vals)
        best = None
        for size in range(1, n + 1):
            feas = [c for c in itertools.combinations(range(n), size)
                    if sum(vals[i] for i in c) >= target]
            if feas:
                best = feas
                break
        got, _, fl = _select1(row, p)
        if fl & oracle.ROW_NEAR_BOUNDARY:
            continue
        # with distinct values the set of the `size` largest entries is feasible, and it is
        # the one the threshold form returns; it must be among the minimum-cardinality sets
        assert tuple(got.tolist()) in best, (row, p)
        assert len(got) == len(best[0])
        top = tuple(sorted(np.argsort(-row.astype(np.float64), kind="stable")[: len(got)].tolist()))
        assert tuple(got.tolist()) == top
        checked += 1
    assert checked >= 40


def test_geometric_row_closed_form():
    """a_j = r^j: the first k entries carry (1 - r^k)/(1 - r^n) of the mass."""
    for r_, n, p in [(0.5, 20, 0.9), (0.8, 64, 0.95), (0.97, 512, 0.9), (0.999, 4096, 0.8),
                     (0.9, 100, 0.5), (0.99, 2000, 0.99)]:
        row = np.float32(r_) ** np.arange(n, dtype=np.float32)
        row = row.astype(np.float32)
        # exact ratio of consecutive stored values differs slightly from r_: count by exact sums
        vals = [Fraction(float(x)) for x in row]
        tot = sum(vals)
        acc, k = Fraction(0), 0
        while acc < Fraction(float(np.float32(p))) * tot:
            acc += vals[k]
            k += 1
        k_formula = math.ceil(math.log(1 - p * (1 - r_ ** n)) / math.log(r_))
        got, tau, fl = _select1(row, p)
        if fl & oracle.ROW_NEAR_BOUNDARY:
            continue
        assert got.tolist() == list(range(k)), (r_, n, p)
        assert abs(k - k_formula) <= 1            # the real-valued formula, up to fp32 storage of r^j
        assert tau == float(row[k - 1])


def test_two_level_rows():
    """k heavy entries a and m light entries b < a: either exactly the heavy ones or everything."""
    rng = np.random.default_rng(5)
    for _ in range(50):
        k, m = int(rng.integers(1, 20)), int(rng.integers(1, 200))
        a, b = 8.0, float(2.0 ** -int(rng.integers(0, 6)))
        row = np.array([a] * k + [b] * m, dtype=np.float32)
        perm = rng.permutation(k + m)
        row = row[perm]
        p = float(np.float32(rng.uniform(0.01, 1.0)))
        heavy_mass, S = a * k, a * k + b * m      # exact in fp64
        got, tau, fl = _select1(row, p)
        if abs(heavy_mass - p * S) <= 1e-5 * S:
            continue
        if p * S <= heavy_mass:
            assert sorted(got.tolist()) == sorted(np.nonzero(row == a)[0].tolist())
            assert tau == a
        else:
            assert got.tolist() == list(range(k + m))
            assert tau == b


def _rows(seed, rows, n):
    rng = np.random.default_rng(seed)
    return W.draft_probs(rng, rows, n, recency_len=min(32, n), spike_frac=0.02)


def test_definition_properties():
    """What Eq. 8 + the threshold form imply, checked with exactly rounded sums (math.fsum)."""
    probs = _rows(3, 24, 777)
    for p in (0.3, 0.9, 0.97, 1.0):
        res = oracle.topp_select(probs, p)
        for r in range(probs.shape[0]):
            row = probs[r].astype(np.float64)
            sel = res.row_set(r)
            tau = float(res.tau[r])
            assert tau in row                                     # tau* is a row value
            assert np.array_equal(sel, np.nonzero(row >= tau)[0])  # threshold form, ascending
            S = math.fsum(row)
            target = float(np.float32(p)) * S
            m_incl = math.fsum(row[row >= tau])
            m_excl = math.fsum(row[row > tau])
            if res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
                continue
            assert m_incl >= target        # feasible
            assert m_excl < target         # dropping the tie group at tau* is not
            assert abs(res.diag[r, 2] - m_incl) <= 1e-12 * S
            assert abs(res.diag[r, 3] - m_excl) <= 1e-12 * S
            assert abs(res.diag[r, 0] - S) <= 1e-12 * S


def test_p_one_keeps_all_positive_and_tiny_p_keeps_argmax():
    probs = _rows(4, 8, 500)
    probs[2, 10:20] = 0.0
    res = oracle.topp_select(probs, 1.0)
    for r in range(8):
        assert np.array_equal(res.row_set(r), np.nonzero(probs[r] > 0)[0])
    res = oracle.topp_select(probs, 1e-7)
    for r in range(8):
        assert np.array_equal(res.row_set(r), np.nonzero(probs[r] == probs[r].max())[0])


def test_monotone_in_p_permutation_and_scaling():
    probs = _rows(6, 6, 640)
    prev = None
    for p in (0.2, 0.5, 0.8, 0.9, 0.95, 0.99, 1.0):
        res = oracle.topp_select(probs, p)
        sets = [set(res.row_set(r).tolist()) for r in range(6)]
        if prev is not None:
            assert all(a <= b for a, b in zip(prev, sets))
        prev = sets
    rng = np.random.default_rng(0)
    perm = rng.permutation(640)
    a = oracle.topp_select(probs, 0.9)
    b = oracle.topp_select(probs[:, perm], 0.9)
    c = oracle.topp_select(probs * np.float32(2.0 ** -7), 0.9)     # exact rescaling
    for r in range(6):
        if a.flags[r] & oracle.ROW_NEAR_BOUNDARY:
            continue
        assert set(perm[b.row_set(r)].tolist()) == set(a.row_set(r).tolist())
        assert np.array_equal(c.row_set(r), a.row_set(r))
        assert c.tau[r] == a.tau[r] * np.float32(2.0 ** -7)


def test_row_lengths_and_invalid_rows():
    probs = _rows(8, 5, 300)
    lens = np.array([300, 17, 1, 0, 250], dtype=np.int32)
    probs[4, 100] = np.nan
    res = oracle.topp_select(probs, 0.9, lens)
    assert (res.row_set(1) < 17).all() and res.counts[1] > 0
    ref = oracle.topp_select(probs[1:2, :17].copy(), 0.9)
    assert np.array_equal(res.row_set(1), ref.row_set(0))
    assert res.row_set(2).tolist() == [0]
    assert res.flags[3] & oracle.ROW_INVALID and res.counts[3] == 0
    assert res.flags[4] & oracle.ROW_INVALID and res.counts[4] == 0
    bad = np.zeros((3, 8), dtype=np.float32)
    bad[1, 3] = -1.0
    bad[2, :] = 0.125
    bad[2, 5] = np.inf
    res = oracle.topp_select(bad, 0.5)
    assert all(res.flags[r] & oracle.ROW_INVALID for r in range(3))     # zero sum, negative, inf
    with pytest.raises(ValueError):
        oracle.topp_select(probs, 0.0)
    with pytest.raises(ValueError):
        oracle.topp_select(probs, 1.5)


def test_numpy_sort_route_agrees():
    """A second, separately written textbook route: argsort + cumsum in numpy."""
    probs = _rows(9, 16, 2048)
    for p in (0.9, 0.95):
        res = oracle.topp_select(probs, p)
        for r in range(16):
            if res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
                continue
            row = probs[r].astype(np.float64)
            order = np.argsort(-row, kind="stable")
            cs = np.cumsum(row[order])
            kk = int(np.searchsorted(cs, float(np.float32(p)) * cs[-1], side="left"))
            thr = row[order[kk]]
            assert np.array_equal(res.row_set(r), np.nonzero(row >= thr)[0])


def test_algorithm2_bisection_cross_check():
    """Algorithm 2 converges to the same set; with few iterations it over-selects.

    Invariant of the loop: theta_low always keeps mass >= target and theta_high never
    does, so tau* lies in [theta_low, theta_high) ... and the bracket halves each step.
    """
    probs = _rows(10, 12, 1500)
    for p in (0.8, 0.95):
        res = oracle.topp_select(probs, p)
        for r in range(12):
            row = probs[r]
            tau = float(res.tau[r])
            mx = float(row.max())
            for iters in (10, 60):
                lo, hi, mid = oracle.nucleus_bisection(row, float(np.float32(p)), iters)
                assert hi - lo <= mx * 2.0 ** -iters + 2 * np.spacing(hi)   # fp64 floor at 60 steps
                if res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
                    continue
                assert lo <= tau
                assert hi > tau or hi == mx
                got = np.nonzero(row.astype(np.float64) >= lo)[0]
                want = res.row_set(r)
                assert set(want.tolist()) <= set(got.tolist())          # never under-selects
                if iters == 60:
                    assert np.array_equal(got, want)                    # converged: same set


def test_ten_iteration_overselection_is_reported_not_asserted():
    """Context for the exact-threshold reading: 10 halvings of [0, max] cannot resolve
    thresholds below max/1024, so long rows with a sink keep far more than the exact set."""
    rng = np.random.default_rng(2)
    probs = W.draft_probs(rng, 4, 8192)
    res = oracle.topp_select(probs, 0.95)
    ratios = []
    for r in range(4):
        lo, _, _ = oracle.nucleus_bisection(probs[r], float(np.float32(0.95)), 10)
        ratios.append(int((probs[r].astype(np.float64) >= lo).sum()) / int(res.counts[r]))
    assert all(x >= 1.0 for x in ratios)
