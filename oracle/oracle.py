"""ctypes front end of the C oracle: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from . import build as _build

ROW_INVALID = 1
ROW_NEAR_BOUNDARY = 2

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = C.CDLL(path)
        lib.oracle_set_threads.restype = C.c_int
        lib.oracle_set_threads.argtypes = [C.c_int]
        lib.oracle_topp_select.restype = C.c_int
        lib.oracle_topp_select.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_float,
                                           C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p]
        lib.oracle_nucleus_bisection.restype = C.c_int
        lib.oracle_nucleus_bisection.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_int,
                                                 C.POINTER(C.c_double), C.POINTER(C.c_double),
                                                 C.POINTER(C.c_double)]
        lib.oracle_masked_attention.restype = C.c_int
        lib.oracle_masked_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                C.c_void_p, C.c_void_p, C.c_double,
                                                C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_masked_attention_tail.restype = C.c_int
        lib.oracle_masked_attention_tail.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                     C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double,
                                                     C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_bisection_select.restype = C.c_int
        lib.oracle_bisection_select.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_float, C.c_int,
                                                C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_chunk_masses.restype = C.c_int
        lib.oracle_chunk_masses.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        _lib = lib
    return _lib


def set_threads(t: int = 0) -> int:
    """Set (t > 0) and return the number of OpenMP threads the oracle uses."""
    return int(_load().oracle_set_threads(int(t)))


@dataclass
class SelectResult:
    indices: np.ndarray     # [rows, n] int32; row r valid on [:counts[r]], ascending
    counts: np.ndarray      # [rows] int32
    tau: np.ndarray         # [rows] float32
    flags: np.ndarray       # [rows] uint32 (ROW_* bits)
    diag: np.ndarray        # [rows, 4] float64: S, target, mass{>= tau}, mass{> tau}

    def row_set(self, r: int) -> np.ndarray:
        return self.indices[r, : self.counts[r]]

    def mask(self) -> np.ndarray:
        """[rows, n] uint8 membership mask."""
        m = np.zeros(self.indices.shape, dtype=np.uint8)
        for r in range(m.shape[0]):
            m[r, self.row_set(r)] = 1
        return m


def topp_select(probs: np.ndarray, top_p: float, lens: Optional[np.ndarray] = None) -> SelectResult:
    """probs [rows, n] float32; lens [rows] (default: n for every row)."""
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    assert probs.ndim == 2
    rows, n = probs.shape
    lens = (np.full(rows, n, dtype=np.int32) if lens is None
            else np.ascontiguousarray(lens, dtype=np.int32))
    assert lens.shape == (rows,) and (lens <= n).all()
    idx = np.full((rows, max(n, 1)), -1, dtype=np.int32)
    counts = np.zeros(rows, dtype=np.int32)
    tau = np.zeros(rows, dtype=np.float32)
    flags = np.zeros(rows, dtype=np.uint32)
    diag = np.zeros((rows, 4), dtype=np.float64)
    rc = _load().oracle_topp_select(probs.ctypes.data, n, rows, lens.ctypes.data, float(top_p),
                                    idx.ctypes.data, idx.shape[1], counts.ctypes.data,
                                    tau.ctypes.data, flags.ctypes.data, diag.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_topp_select failed with {rc} (top_p must be in (0, 1])")
    return SelectResult(idx, counts, tau, flags, diag)


def bisection_select(probs: np.ndarray, top_p: float, iters: int,
                     lens: Optional[np.ndarray] = None) -> SelectResult:
    """Algorithm 2 with `iters` halvings per row (the paper's implementation: 10); set {a >= theta_low}."""
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    rows, n = probs.shape
    lens = np.full(rows, n, dtype=np.int32) if lens is None else np.ascontiguousarray(lens, dtype=np.int32)
    idx = np.full((rows, max(n, 1)), -1, dtype=np.int32)
    counts = np.zeros(rows, dtype=np.int32)
    tau = np.zeros(rows, dtype=np.float32)
    flags = np.zeros(rows, dtype=np.uint32)
    rc = _load().oracle_bisection_select(probs.ctypes.data, n, rows, lens.ctypes.data, float(top_p), int(iters),
                                         idx.ctypes.data, idx.shape[1], counts.ctypes.data, tau.ctypes.data,
                                         flags.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_bisection_select failed with {rc}")
    return SelectResult(idx, counts, tau, flags, np.zeros((rows, 4)))


def chunk_masses(probs: np.ndarray, chunk: int, lens: Optional[np.ndarray] = None) -> np.ndarray:
    """probs [rows, n] float32 -> [rows, ceil(n / chunk)] float32 chunk masses (fp64 sums, rounded once)."""
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    rows, n = probs.shape
    lens = np.full(rows, n, dtype=np.int32) if lens is None else np.ascontiguousarray(lens, dtype=np.int32)
    nc = (n + chunk - 1) // chunk
    mass = np.zeros((rows, nc), dtype=np.float32)
    rc = _load().oracle_chunk_masses(probs.ctypes.data, n, rows, lens.ctypes.data, int(chunk), nc, mass.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_chunk_masses failed with {rc}")
    return mass


def topp_select_chunks(probs: np.ndarray, top_p: float, chunk: int,
                       lens: Optional[np.ndarray] = None) -> SelectResult:
    """Chunk-granular selection: exact top-p over the row of chunk masses.  The result's indices are
    chunk numbers; chunk c stands for positions [c*chunk, min((c+1)*chunk, len))."""
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    rows, n = probs.shape
    lens = np.full(rows, n, dtype=np.int32) if lens is None else np.ascontiguousarray(lens, dtype=np.int32)
    mass = chunk_masses(probs, chunk, lens)
    return topp_select(mass, top_p, lens=(lens + chunk - 1) // chunk)


def chunk_token_mask(res: SelectResult, chunk: int, n: int, lens: Optional[np.ndarray] = None) -> np.ndarray:
    """[rows, n] uint8: the positions the kept chunks stand for."""
    rows = res.counts.shape[0]
    lens = np.full(rows, n, dtype=np.int32) if lens is None else lens
    m = np.zeros((rows, n), dtype=np.uint8)
    for r in range(rows):
        for c in res.row_set(r):
            m[r, c * chunk: min((c + 1) * chunk, int(lens[r]))] = 1
    return m


@dataclass
class UnionResult:
    indices: np.ndarray     # [B*H_kv, n] int32; row r valid on [:counts[r]], ascending
    counts: np.ndarray      # [B*H_kv] int32
    flags: np.ndarray       # [B*H_kv] uint32: INVALID if every member row is invalid, NEAR_BOUNDARY if any valid one is
    members: SelectResult   # the per-(b, draft head, step) selections the union was taken over

    def row_set(self, r: int) -> np.ndarray:
        return self.indices[r, : self.counts[r]]

    def mask(self) -> np.ndarray:
        m = np.zeros(self.indices.shape, dtype=np.uint8)
        for r in range(m.shape[0]):
            m[r, self.row_set(r)] = 1
        return m


def topp_select_union(probs: np.ndarray, top_p: float, H_kv: int,
                      lens: Optional[np.ndarray] = None) -> UnionResult:
    """Algorithm 2 as a whole: top-p selection of every draft step's row, then the union of the sets.

    probs [B, H_draft, S, n] float32: the draft attention row of every (sequence, draft head,
    speculative step).  Draft heads h*H_draft/H_kv .. (h+1)*H_draft/H_kv - 1 feed kv head h, and the
    union runs over their rows as well as over the S steps.  lens [B]: common valid length.
    """
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    assert probs.ndim == 4
    B, H_d, S, n = probs.shape
    assert H_d % H_kv == 0
    per = H_d // H_kv
    lens = np.full(B, n, dtype=np.int32) if lens is None else np.ascontiguousarray(lens, dtype=np.int32)
    members = topp_select(probs.reshape(B * H_d * S, n), top_p, lens=np.repeat(lens, H_d * S))
    R = B * H_kv
    idx = np.full((R, max(n, 1)), -1, dtype=np.int32)
    counts = np.zeros(R, dtype=np.int32)
    flags = np.zeros(R, dtype=np.uint32)
    for b in range(B):
        for h in range(H_kv):
            r = b * H_kv + h
            kept = set()
            all_invalid, any_near = True, False
            for hd in range(h * per, (h + 1) * per):
                for s in range(S):
                    m = (b * H_d + hd) * S + s
                    if members.flags[m] & ROW_INVALID:
                        continue
                    all_invalid = False
                    any_near = any_near or bool(members.flags[m] & ROW_NEAR_BOUNDARY)
                    kept.update(int(j) for j in members.row_set(m))     # T <- T u T_s
            out = sorted(kept)
            counts[r] = len(out)
            idx[r, : len(out)] = out
            flags[r] = (ROW_INVALID if all_invalid else 0) | (ROW_NEAR_BOUNDARY if any_near else 0)
    return UnionResult(idx, counts, flags, members)


def nucleus_bisection(row: np.ndarray, p: float, iters: int):
    """Algorithm 2's bisection on one row; returns (theta_low, theta_high, theta_mid)."""
    row = np.ascontiguousarray(row, dtype=np.float32)
    lo, hi, mid = C.c_double(), C.c_double(), C.c_double()
    _load().oracle_nucleus_bisection(row.ctypes.data, row.size, float(p), int(iters),
                                     C.byref(lo), C.byref(hi), C.byref(mid))
    return lo.value, hi.value, mid.value


def masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray,
                     *, bf16: bool = False, f16: bool = False, lens: Optional[np.ndarray] = None,
                     sm_scale: Optional[float] = None,
                     which: Optional[Sequence[Sequence[int]]] = None,
                     k_new: Optional[np.ndarray] = None, v_new: Optional[np.ndarray] = None):
    """Masked dense attention in fp64.

    q [B,H_q,T,d], k/v [B,H_kv,n,d]: float32 arrays, or uint16 bit patterns
    (bf16 when bf16=True, IEEE half when f16=True).  mask [B,H_kv,n] (nonzero = selected).
    k_new/v_new [B,H_kv,T,d] (optional): the new tokens' keys and values;
    query t also attends to new tokens 0..t, whatever the mask says.
    which: optional list of (b, h_q, t) rows; default all, returned as
    out [B,H_q,T,d] / lse [B,H_q,T].  With `which`, out is [len(which), d].
    """
    assert not (bf16 and f16)
    want = np.uint16 if (bf16 or f16) else np.float32
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    assert q.dtype == want and k.dtype == want and v.dtype == want
    B, H_q, T, d = q.shape
    _, H_kv, n, _ = k.shape
    assert k.shape == v.shape == (B, H_kv, n, d)
    assert (k_new is None) == (v_new is None)
    if k_new is not None:
        k_new, v_new = np.ascontiguousarray(k_new), np.ascontiguousarray(v_new)
        assert k_new.dtype == want and v_new.dtype == want
        assert k_new.shape == v_new.shape == (B, H_kv, T, d)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.shape == (B, H_kv, n)
    lens = (np.full(B, n, dtype=np.int32) if lens is None
            else np.ascontiguousarray(lens, dtype=np.int32))
    scale = float(1.0 / np.sqrt(np.float64(d))) if sm_scale is None else float(sm_scale)
    full = which is None
    if full:
        which_a = np.array([(b, h, t) for b in range(B) for h in range(H_q) for t in range(T)],
                           dtype=np.int32)
    else:
        which_a = np.ascontiguousarray(which, dtype=np.int32).reshape(-1, 3)
    rows = which_a.shape[0]
    out = np.zeros((rows, d), dtype=np.float64)
    lse = np.zeros(rows, dtype=np.float64)
    rc = _load().oracle_masked_attention_tail(q.ctypes.data, k.ctypes.data, v.ctypes.data, 1 if bf16 else (2 if f16 else 0),
                                              B, H_q, H_kv, T, d, n, mask.ctypes.data, lens.ctypes.data,
                                              None if k_new is None else k_new.ctypes.data,
                                              None if v_new is None else v_new.ctypes.data,
                                              scale, which_a.ctypes.data, rows,
                                              out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_masked_attention_tail failed with {rc}")
    if full:
        return out.reshape(B, H_q, T, d), lse.reshape(B, H_q, T)
    return out, lse
