"""Seeded synthetic inputs for the top-p select + sparse decode attention path.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no threshold search, no selection, no attention) and is the one piece of
code that both the CPU oracle's tests and the HIP path's tests/bench share.

The paper evaluates on real draft-model attention rows (PG-19 / LongBench
text through TinyLlama -> Llama-2, Section 4).  Neither the models nor the
datasets are available offline, so the rows below are stand-ins with the
structure decode-time attention rows are known to have: an attention sink at
position 0, a recency band at the end of the context, a log-normal bulk and a
sparse set of strongly attended positions.

Every array is a numpy array.  bf16 tensors are returned as float32 arrays
whose values are exactly representable in bf16, next to their raw uint16 bit
patterns, so that the oracle (which reads the bits) and the GPU path (which
gets the same bits as a torch.bfloat16 tensor) see identical inputs.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

PAGE_SIZE = 16


# --------------------------------------------------------------------------
# dtype helpers (input preparation only)
# --------------------------------------------------------------------------
def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 array holding the same values."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# draft attention rows
# --------------------------------------------------------------------------
def draft_probs(
    rng: np.random.Generator,
    rows: int,
    n: int,
    *,
    lens: Optional[np.ndarray] = None,
    sigma: float = 2.0,
    sink: float = 6.0,
    recency_boost: float = 3.0,
    recency_len: int = 64,
    spike_frac: float = 0.01,
    spike_max: float = 4.0,
    spike_zipf: float = 1.1,
    student_t_nu: Optional[float] = None,
    logit_clip: Optional[float] = None,
) -> np.ndarray:
    """[rows, n] float32 rows, each the softmax of synthetic draft logits.

    logits = sigma * z  (z ~ N(0,1), or Student-t(nu) when student_t_nu is set)
             + sink at position 0
             + recency_boost on the last recency_len valid positions
             + spike_max * k**(-spike_zipf) on the k-th of
               round(spike_frac * len) random positions (k = 1, 2, ...).
    Positions >= lens[r] get probability exactly 0.
    """
    out = np.zeros((rows, n), dtype=np.float32)
    for r in range(rows):
        ln = int(n if lens is None else lens[r])
        if ln == 0:
            continue
        if student_t_nu is None:
            z = rng.standard_normal(ln)
        else:
            z = rng.standard_t(student_t_nu, ln)
        logit = sigma * z
        if logit_clip is not None:
            np.clip(logit, -logit_clip, logit_clip, out=logit)
        logit[0] += sink
        logit[max(0, ln - recency_len):ln] += recency_boost
        k = int(round(spike_frac * ln))
        if k > 0 and spike_max > 0.0:
            pos = rng.choice(ln, size=k, replace=False)
            logit[pos] += spike_max * np.arange(1, k + 1, dtype=np.float64) ** (-spike_zipf)
        logit -= logit.max()
        e = np.exp(logit)
        out[r, :ln] = (e / e.sum()).astype(np.float32)
    return out


def draft_step_probs(
    rng: np.random.Generator,
    B: int,
    H_draft: int,
    S: int,
    n: int,
    *,
    lens: Optional[np.ndarray] = None,
    step_sigma: float = 0.7,
    **kw,
) -> np.ndarray:
    """[B, H_draft, S, n] float32: the draft attention rows of S consecutive speculative steps.

    The S rows of one (sequence, head) share their logits (drawn as in draft_probs) up to an
    independent N(0, step_sigma^2) perturbation per step and position, so consecutive steps attend
    to mostly, but not exactly, the same positions.  Positions >= lens[b] hold exactly 0 (the
    draft's attention to its own speculative tokens is not part of the verifier's cache, so a
    row's mass over the cache may be below 1).
    """
    sigma = kw.pop("sigma", 2.0)
    sink = kw.pop("sink", 6.0)
    recency_boost = kw.pop("recency_boost", 3.0)
    recency_len = kw.pop("recency_len", 64)
    spike_frac = kw.pop("spike_frac", 0.01)
    spike_max = kw.pop("spike_max", 4.0)
    spike_zipf = kw.pop("spike_zipf", 1.1)
    assert not kw, f"unknown arguments {sorted(kw)}"
    out = np.zeros((B, H_draft, S, n), dtype=np.float32)
    for b in range(B):
        ln = int(n if lens is None else lens[b])
        if ln == 0:
            continue
        for h in range(H_draft):
            base = sigma * rng.standard_normal(ln)
            base[0] += sink
            base[max(0, ln - recency_len):ln] += recency_boost
            k = int(round(spike_frac * ln))
            if k > 0 and spike_max > 0.0:
                pos = rng.choice(ln, size=k, replace=False)
                base[pos] += spike_max * np.arange(1, k + 1, dtype=np.float64) ** (-spike_zipf)
            for s_ in range(S):
                logit = base + step_sigma * rng.standard_normal(ln)
                logit -= logit.max()
                e = np.exp(logit)
                # the step's own s_ speculative tokens take a little of the mass (not part of the cache)
                out[b, h, s_, :ln] = (e / (e.sum() * (1.0 + 0.02 * s_))).astype(np.float32)
    return out


# --------------------------------------------------------------------------
# workload container
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    H_q: int
    H_kv: int
    T: int                      # gamma + 1 verifier queries
    d: int
    n: int                      # n_max (padded context length)
    top_p: float
    dtype: str                  # "f32" | "bf16" | "f16"
    probs: np.ndarray           # [B, H_kv, n] float32
    q: np.ndarray               # [B, H_q, T, d] float32 (bf16-representable when dtype == "bf16")
    k: np.ndarray               # [B, H_kv, n, d] float32, logical (un-paged) order
    v: np.ndarray
    seq_lens: Optional[np.ndarray] = None      # [B] int32 or None
    page_table: Optional[np.ndarray] = None    # [B, max_pages] int32 or None
    n_pool_pages: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.H_q // self.H_kv

    def row_lens(self) -> np.ndarray:
        """[B*H_kv] int32 valid length of every selection row."""
        if self.seq_lens is None:
            return np.full(self.B * self.H_kv, self.n, dtype=np.int32)
        return np.repeat(self.seq_lens.astype(np.int32), self.H_kv)

    def paged_pool(self, x: np.ndarray) -> np.ndarray:
        """Scatter logical [B, H_kv, n, d] into the pool [pages, H_kv, PAGE_SIZE, d]."""
        assert self.page_table is not None
        pool = np.zeros((self.n_pool_pages, self.H_kv, PAGE_SIZE, self.d), dtype=x.dtype)
        for b in range(self.B):
            ln = int(self.n if self.seq_lens is None else self.seq_lens[b])
            for p in range((ln + PAGE_SIZE - 1) // PAGE_SIZE):
                lo = p * PAGE_SIZE
                hi = min(lo + PAGE_SIZE, ln)
                pool[self.page_table[b, p], :, : hi - lo, :] = x[b, :, lo:hi, :]
        return pool


def _qkv(rng, B, H_q, H_kv, T, d, n, dtype):
    q = rng.standard_normal((B, H_q, T, d), dtype=np.float32)
    k = rng.standard_normal((B, H_kv, n, d), dtype=np.float32)
    v = rng.standard_normal((B, H_kv, n, d), dtype=np.float32)
    if dtype == "bf16":
        q, k, v = (bf16_bits_to_f32(round_to_bf16_bits(a)).reshape(a.shape) for a in (q, k, v))
    elif dtype == "f16":
        q, k, v = (a.astype(np.float16).astype(np.float32) for a in (q, k, v))
    return q, k, v


def tiny_f32(seed: int = 0, n: int = 1024, B: int = 1, H: int = 8, T: int = 5, d: int = 64,
             top_p: float = 0.9) -> Workload:
    """Tiny fp32 MHA instance: sink + 32-position recency band, no spikes."""
    rng = np.random.default_rng(seed)
    probs = draft_probs(rng, B * H, n, recency_len=32, spike_frac=0.0).reshape(B, H, n)
    q, k, v = _qkv(rng, B, H, H, T, d, n, "f32")
    return Workload("tiny_f32", B, H, H, T, d, n, top_p, "f32", probs, q, k, v)


def llama8b_layer(seed: int = 0, B: int = 1, n: int = 8192, top_p: float = 0.95, H_q: int = 32,
                  H_kv: int = 8, T: int = 5, d: int = 128, dtype: str = "bf16",
                  with_kv: bool = True) -> Workload:
    """One Llama-3-8B-shaped layer: GQA group 4, d = 128, bf16 Q/K/V.

    with_kv=False leaves q/k/v as empty arrays (callers that draw K/V on the
    device for the large configurations only need the draft rows from here).
    """
    rng = np.random.default_rng(seed)
    probs = draft_probs(rng, B * H_kv, n).reshape(B, H_kv, n)
    if with_kv:
        q, k, v = _qkv(rng, B, H_q, H_kv, T, d, n, dtype)
    else:
        q = k = v = np.zeros((0,), dtype=np.float32)
    return Workload("llama8b_layer", B, H_q, H_kv, T, d, n, top_p, dtype, probs, q, k, v)


def long_context(seed: int = 0, B: int = 4, n: int = 131072, top_p: float = 0.9, H_q: int = 32,
                 H_kv: int = 8, T: int = 5, d: int = 128, logit_clip: Optional[float] = None,
                 with_kv: bool = True) -> Workload:
    """Heavy-tailed draft logits: scale-2 Student-t(nu=3) + sink + recency.

    Read literally the unclipped t(3) logits put almost all mass on one or two
    positions; logit_clip gives the labelled supplementary variant.
    """
    rng = np.random.default_rng(seed)
    probs = draft_probs(rng, B * H_kv, n, student_t_nu=3.0, spike_frac=0.0,
                        logit_clip=logit_clip).reshape(B, H_kv, n)
    if with_kv:
        q, k, v = _qkv(rng, B, H_q, H_kv, T, d, n, "bf16")
    else:
        q = k = v = np.zeros((0,), dtype=np.float32)
    w = Workload("long_context", B, H_q, H_kv, T, d, n, top_p, "bf16", probs, q, k, v)
    w.meta["logit_clip"] = logit_clip
    return w


def ragged_paged(seed: int = 0, B: int = 64, len_lo: int = 4096, len_hi: int = 65536,
                 top_p: float = 0.95, H_q: int = 32, H_kv: int = 8, T: int = 5, d: int = 128,
                 with_kv: bool = True, extra_pages: int = 3) -> Workload:
    """Ragged batch over a shared 16-token-paged pool with a random page table."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(len_lo, len_hi + 1, size=B).astype(np.int32)
    n = int(-(-int(lens.max()) // PAGE_SIZE) * PAGE_SIZE)
    pages_per_seq = (lens + PAGE_SIZE - 1) // PAGE_SIZE
    total_pages = int(pages_per_seq.sum()) + extra_pages
    perm = rng.permutation(total_pages).astype(np.int32)
    max_pages = n // PAGE_SIZE
    table = np.full((B, max_pages), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, : pages_per_seq[b]] = perm[at: at + pages_per_seq[b]]
        at += int(pages_per_seq[b])
    probs = draft_probs(rng, B * H_kv, n, lens=np.repeat(lens, H_kv)).reshape(B, H_kv, n)
    if with_kv:
        q, k, v = _qkv(rng, B, H_q, H_kv, T, d, n, "bf16")
        for b in range(B):          # positions past the sequence end hold no data
            k[b, :, lens[b]:, :] = 0.0
            v[b, :, lens[b]:, :] = 0.0
    else:
        q = k = v = np.zeros((0,), dtype=np.float32)
    return Workload("ragged_paged", B, H_q, H_kv, T, d, n, top_p, "bf16", probs, q, k, v,
                    seq_lens=lens, page_table=table, n_pool_pages=total_pages)


def layer_attention_maps(seed: int = 0, m: int = 22, n: int = 32, rows: int = 64, L: int = 2048):
    """Aligned causal attention rows of a draft model with m layers and a verifier with n layers (stand-ins for the
    rows collected on a text corpus): row r sees the first len_r positions; a layer at relative depth t in [0, 1]
    puts weight on the first position (sink, growing with depth), on a recency window (narrowing with depth) and
    on a few content positions shared by both models, over layer-specific noise.  Layers of the two models at the
    same relative depth therefore resemble each other.  Returns (attn_draft [m, rows, L], attn_verifier
    [n, rows, L]) float32, rows summing to 1 over the visible positions and 0 beyond."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(min(L, max(8, L // 8)), L + 1, size=rows)
    content = [rng.choice(int(lens[r]), size=min(8, int(lens[r])), replace=False) for r in range(rows)]

    def model(layers):
        out = np.zeros((layers, rows, L), dtype=np.float64)
        for i in range(layers):
            t = i / max(layers - 1, 1)
            for r in range(rows):
                ln = int(lens[r])
                logit = 0.5 * rng.standard_normal(ln)
                logit[0] += 2.0 + 4.0 * t
                width = int(min(ln, max(2, round(ln * (0.25 - 0.2 * t)))))
                logit[ln - width:] += 2.0
                logit[content[r]] += 1.0 + 3.0 * np.sin(np.pi * t)
                e = np.exp(logit - logit.max())
                out[i, r, :ln] = e / e.sum()
        return out.astype(np.float32)

    return model(m), model(n)
