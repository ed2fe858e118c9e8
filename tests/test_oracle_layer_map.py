"""Pins of the layer-mapping oracle (Section 3.3, Eq. 4; Appendix B, Algorithm 3): hand-worked values, closed forms,
a library routine, exhaustive search, and Algorithm 3's own three-transition table written out separately."""
import os

import numpy as np
import pytest
from scipy.special import rel_entr

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layer_map_hand.txt")


def _cases(kind):
    for ln in open(GOLDEN):
        ln = ln.strip()
        if not ln or ln.startswith("#"):
            continue
        parts = [p.strip() for p in ln.split("|")]
        if parts[0] == kind:
            yield parts[1:]


def test_hand_worked_divergences():
    n = 0
    for v, d, want in _cases("kl"):
        av = np.array([[[float(x) for x in v.split()]]])
        ad = np.array([[[float(x) for x in d.split()]]])
        S = oracle.layer_similarity(ad, av)
        assert S.shape == (1, 1)
        if want == "inf":
            assert S[0, 0] == -np.inf
        else:
            assert abs(-S[0, 0] - float(want)) <= 1e-15
        n += 1
    assert n == 6


def test_hand_worked_alignments():
    n = 0
    for dims, vals, want, f_want in _cases("map"):
        m, nn = (int(x) for x in dims.split())
        S = np.array([float(x) for x in vals.split()]).reshape(m, nn)
        best, all_f = oracle.layer_map_exhaustive(S)
        f, val = oracle.layer_map(S)
        assert best == float(want) and val == float(want)
        assert tuple(int(x) for x in f_want.split()) in all_f
        assert tuple(int(x) for x in f) in all_f
        n += 1
    assert n == 7


def _rand_rows(rng, layers, rows, L, zeros=False):
    a = rng.gamma(0.3, size=(layers, rows, L))
    if zeros:
        a[rng.random(a.shape) < 0.2] = 0.0
        a[..., 0] += 1e-3                                   # no empty rows
    return a / a.sum(axis=-1, keepdims=True)


def test_similarity_against_a_library_routine_and_its_properties():
    rng = np.random.default_rng(0)
    ad, av = _rand_rows(rng, 3, 4, 17), _rand_rows(rng, 2, 4, 17, zeros=True)
    S = oracle.layer_similarity(ad, av)
    for i in range(3):
        for j in range(2):
            want = -np.mean([rel_entr(av[j, r], ad[i, r]).sum() for r in range(4)])
            assert abs(S[i, j] - want) <= 1e-13 * max(1.0, abs(want))
    assert (S < 0).all()                                    # Gibbs: the divergence of different rows is positive
    # the operands are not interchangeable (verifier first)
    assert abs(oracle.layer_similarity(ad[:2], av)[1, 0] - oracle.layer_similarity(av, ad[:2])[0, 1]) > 1e-3
    # a layer compared with itself
    assert np.allclose(np.diag(oracle.layer_similarity(ad, ad)), 0.0, atol=1e-15)
    # mean over rows: doubling the rows changes nothing; the two halves average
    twice = oracle.layer_similarity(np.concatenate([ad, ad], axis=1), np.concatenate([av, av], axis=1))
    assert np.allclose(twice, S, rtol=1e-14)
    halves = 0.5 * (oracle.layer_similarity(ad[:, :2], av[:, :2]) + oracle.layer_similarity(ad[:, 2:], av[:, 2:]))
    assert np.allclose(halves, S, rtol=1e-13)
    # a permutation of the positions, applied to both models, changes nothing (up to summation order)
    perm = rng.permutation(17)
    assert np.allclose(oracle.layer_similarity(ad[..., perm], av[..., perm]), S, rtol=1e-13)
    # against the uniform row: ln L - entropy
    uni = np.full((1, 4, 17), 1.0 / 17)
    ent = -(np.where(av > 0, av * np.log(np.where(av > 0, av, 1.0)), 0.0)).sum(axis=-1)
    assert np.allclose(-oracle.layer_similarity(uni, av)[0], (np.log(17) - ent).mean(axis=1), rtol=1e-13)
    # the vectorised form is the same sum
    assert np.allclose(oracle.layer_similarity_fast(ad, av), S, rtol=1e-13)


def test_draft_zero_under_verifier_mass_is_minus_infinity():
    ad = np.array([[[0.5, 0.5, 0.0]], [[0.25, 0.25, 0.5]]])
    av = np.array([[[0.5, 0.25, 0.25]], [[0.5, 0.5, 0.0]]])
    S = oracle.layer_similarity(ad, av)
    assert S[0, 0] == -np.inf and np.isfinite(S[1, 0]) and np.isfinite(S[0, 1]) and np.isfinite(S[1, 1])
    assert np.array_equal(oracle.layer_similarity_fast(ad, av) == -np.inf, S == -np.inf)


def _algorithm3(S):
    """Appendix B, Algorithm 3, step by step: distance D = -S, table dp over (draft layers + 1) x (verifier layers
    + 1) with dp[0][0] = 0 and infinity elsewhere, three transitions, minimum of the last column."""
    m, n = S.shape
    D = -S
    dp = np.full((m + 1, n + 1), np.inf)
    dp[0, 0] = 0.0
    for i in range(1, m + 1):
        for j in range(1, n + 1):
            cost = D[i - 1, j - 1]
            diagonal = dp[i - 1, j - 1] + cost
            left = dp[i, j - 1] + cost
            above = dp[: i + 1, j - 1].min() + cost
            dp[i, j] = min(diagonal, left, above)
    return -dp[1:, n].min()


@pytest.mark.parametrize("seed", range(40))
def test_recurrence_against_exhaustive_search_and_algorithm_3(seed):
    rng = np.random.default_rng(seed)
    m, n = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    S = -rng.gamma(1.0, size=(m, n)) if seed % 3 else np.round(rng.normal(size=(m, n)), 0)      # ties in every third case
    best, all_f = oracle.layer_map_exhaustive(S)
    f, val = oracle.layer_map(S)
    assert abs(val - best) <= 1e-12
    assert all(f[j] <= f[j + 1] for j in range(n - 1)) and 0 <= f.min() and f.max() < m
    assert abs(sum(S[f[j], j] for j in range(n)) - best) <= 1e-12
    assert tuple(int(x) for x in f) in all_f
    assert abs(_algorithm3(S) - best) <= 1e-12


def test_dominant_diagonal_gives_the_identity_and_a_dominant_row_a_constant_map():
    rng = np.random.default_rng(5)
    S = -rng.gamma(1.0, size=(6, 6)) - 10.0
    S[np.arange(6), np.arange(6)] = -0.1
    f, _ = oracle.layer_map(S)
    assert list(f) == [0, 1, 2, 3, 4, 5]
    S = -rng.gamma(1.0, size=(5, 7)) - 10.0
    S[2] = -0.1
    f, _ = oracle.layer_map(S)
    assert list(f) == [2] * 7
