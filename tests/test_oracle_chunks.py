"""Pins for the oracle's chunk-granular selection (chunk masses + exact top-p over them; CPU only)."""
from fractions import Fraction

import numpy as np

import oracle


def test_hand_worked_chunks():
    # chunks of 4: masses 0.5 | 0.125 | 0.375 (last chunk is partial: length 10); all sums are exact in binary
    row = np.array([[0.25, 0.125, 0.0625, 0.0625, 0.03125, 0.03125, 0.03125, 0.03125, 0.25, 0.125, 9.0, 9.0]],
                   dtype=np.float32)
    lens = np.array([10], dtype=np.int32)
    mass = oracle.chunk_masses(row, 4, lens)
    assert mass.tolist() == [[0.5, 0.125, 0.375]]
    # p = 0.8: 0.5 < 0.8, 0.5 + 0.375 >= 0.8 -> chunks {0, 2}
    res = oracle.topp_select_chunks(row, 0.8, 4, lens)
    assert list(res.row_set(0)) == [0, 2]
    tok = oracle.chunk_token_mask(res, 4, 12, lens)
    assert tok[0].tolist() == [1, 1, 1, 1, 0, 0, 0, 0, 1, 1, 0, 0]
    # p = 0.5 sits exactly on the first chunk: kept alone, and flagged as a boundary row
    res = oracle.topp_select_chunks(row, 0.5, 4, lens)
    assert list(res.row_set(0)) == [0] and res.flags[0] & oracle.ROW_NEAR_BOUNDARY


def test_masses_are_the_correctly_rounded_exact_sums():
    rng = np.random.default_rng(0)
    probs = rng.dirichlet(np.full(200, 0.3), size=3).astype(np.float32)
    mass = oracle.chunk_masses(probs, 16)
    for r in range(3):
        for c in range(13):
            exact = sum(Fraction(float(x)) for x in probs[r, 16 * c: 16 * c + 16])
            # fp64 holds these sums of 16 fp32 values exactly (they span far fewer than 29 binades here)
            assert Fraction(float(np.float32(float(exact)))) == Fraction(float(mass[r, c]))
        assert abs(float(mass[r].astype(np.float64).sum()) - float(probs[r].astype(np.float64).sum())) < 1e-6


def test_chunk_of_one_is_plain_selection():
    rng = np.random.default_rng(1)
    probs = rng.dirichlet(np.full(300, 0.2), size=4).astype(np.float32)
    a = oracle.topp_select_chunks(probs, 0.9, 1)
    b = oracle.topp_select(probs, 0.9)
    assert np.array_equal(a.counts, b.counts) and np.array_equal(a.tau, b.tau)
    for r in range(4):
        assert np.array_equal(a.row_set(r), b.row_set(r))


def test_kept_chunks_hold_the_target_mass_and_are_minimal():
    rng = np.random.default_rng(2)
    probs = rng.dirichlet(np.full(1000, 0.1), size=6).astype(np.float32)
    lens = np.array([1000, 999, 17, 16, 1, 500], dtype=np.int32)
    for r in range(6):
        probs[r, lens[r]:] = 0.0
    res = oracle.topp_select_chunks(probs, 0.9, 16, lens)
    mass = oracle.chunk_masses(probs, 16, lens).astype(np.float64)
    for r in range(6):
        kept = res.row_set(r)
        assert (kept < (lens[r] + 15) // 16).all()
        total, got = mass[r].sum(), mass[r, kept].sum()
        assert got >= 0.9 * total * (1 - 1e-12)
        smallest = mass[r, kept].min()
        if not res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
            assert got - mass[r, kept][mass[r, kept] == smallest].sum() < 0.9 * total     # dropping the tie group fails
        assert (mass[r, np.setdiff1d(np.arange(mass.shape[1]), kept)] < smallest).all()


def test_invalid_entry_makes_the_row_invalid():
    probs = np.full((2, 64), 1 / 64, dtype=np.float32)
    probs[0, 37] = -0.25                     # would hide inside a positive chunk mass
    res = oracle.topp_select_chunks(probs, 0.9, 16)
    assert res.flags[0] & oracle.ROW_INVALID and res.counts[0] == 0
    assert not res.flags[1] & oracle.ROW_INVALID and res.counts[1] == 4
