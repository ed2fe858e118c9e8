"""CPU oracle (test infrastructure) for the offline layer mapping: the similarity of Section 3.3, Eq. 4, and the
monotone alignment of Appendix B (Algorithm 3).  Plain numpy in fp64; small inputs only.

Never imported by the product.  Shares no code with the HIP path.

Readings taken where the paper is silent:
  * Eq. 4 compares two vectors A^v_j, A^d_i in R^L.  A representative data set gives many attention rows per
    layer (heads x queries x samples); the similarity of a layer pair is the mean of Eq. 4 over those rows.
    Rows of the two models are aligned (row r of every layer belongs to the same query of the same text).
  * 0 * log(0 / x) = 0 (positions a causal row cannot see carry no mass in either model);
    a verifier mass on a position where the draft row is exactly 0 makes the divergence infinite (S = -inf).
  * Appendix B states the objective in closed form: f maps verifier layers to draft layers, is non-decreasing,
    and maximises sum_j S[f(j), j].  The oracle is that definition: exhaustive search for tiny sizes, and the
    recurrence best[i][j] = S[i][j] + max_{k <= i} best[k][j-1] (Algorithm 3's "above" transition, which contains
    its "diagonal" and "left" transitions) otherwise.  Several maps can reach the optimum; the value is unique.
"""
from __future__ import annotations

import itertools

import numpy as np


def layer_similarity(attn_draft: np.ndarray, attn_verifier: np.ndarray) -> np.ndarray:
    """attn_draft [m, rows, L], attn_verifier [n, rows, L] (probabilities, any float type) -> S [m, n] fp64,
    S[i, j] = -(1/rows) * sum_r KL(attn_verifier[j, r] || attn_draft[i, r])   (Eq. 4, averaged over rows)."""
    ad = np.asarray(attn_draft, dtype=np.float64)
    av = np.asarray(attn_verifier, dtype=np.float64)
    m, rows, L = ad.shape
    n = av.shape[0]
    assert av.shape[1:] == (rows, L)
    S = np.zeros((m, n), dtype=np.float64)
    for i in range(m):
        for j in range(n):
            kl = 0.0
            for r in range(rows):
                for k in range(L):
                    p, q = av[j, r, k], ad[i, r, k]
                    if p > 0.0:
                        kl += np.inf if q == 0.0 else p * (np.log(p) - np.log(q))
            S[i, j] = -kl / rows
    return S


def layer_similarity_fast(attn_draft: np.ndarray, attn_verifier: np.ndarray) -> np.ndarray:
    """The same sum with numpy array operations (for inputs too large for the loops above)."""
    ad = np.asarray(attn_draft, dtype=np.float64)
    av = np.asarray(attn_verifier, dtype=np.float64)
    m, rows, _ = ad.shape
    n = av.shape[0]
    with np.errstate(divide="ignore", invalid="ignore"):
        lad, lav = np.log(ad), np.log(av)
        S = np.zeros((m, n), dtype=np.float64)
        for i in range(m):
            for j in range(n):
                t = np.where(av[j] > 0.0, av[j] * (lav[j] - lad[i]), 0.0)
                S[i, j] = -t.sum() / rows
    return S


def monotone_maps(m: int, n: int):
    """Every non-decreasing f: {0..n-1} -> {0..m-1}."""
    return itertools.combinations_with_replacement(range(m), n)


def layer_map_exhaustive(S: np.ndarray):
    """Optimum of sum_j S[f(j), j] over all non-decreasing f, by enumeration.  Returns (best value, all optimal f)."""
    S = np.asarray(S, dtype=np.float64)
    m, n = S.shape
    best, arg = -np.inf, []
    for f in monotone_maps(m, n):
        val = sum(S[f[j], j] for j in range(n))
        if val > best:
            best, arg = val, [f]
        elif val == best:
            arg.append(f)
    return best, arg


def layer_map(S: np.ndarray):
    """The same optimum by the recurrence; returns (f [n] int32 with the smallest draft index at every tie, value)."""
    S = np.asarray(S, dtype=np.float64)
    m, n = S.shape
    best = np.full((m, n), -np.inf)
    back = np.zeros((m, n), dtype=np.int64)
    best[:, 0] = S[:, 0]
    for j in range(1, n):
        for i in range(m):
            k = int(np.argmax(best[: i + 1, j - 1]))          # first maximum
            best[i, j] = S[i, j] + best[k, j - 1]
            back[i, j] = k
    i = int(np.argmax(best[:, n - 1]))
    f = np.zeros(n, dtype=np.int32)
    f[n - 1] = i
    for j in range(n - 1, 0, -1):
        i = back[i, j]
        f[j - 1] = i
    return f, float(best[f[n - 1], n - 1])
