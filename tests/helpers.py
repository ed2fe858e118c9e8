"""Shared test helpers: run the HIP path through the C ABI, run the oracle, compare.

The HIP path and the oracle only meet here: both get the same seeded inputs,
and nothing computed by one is ever fed to the other.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

TOL = {"bf16": 2e-3, "f16": 2e-3, "f32": 1e-5}     # max |out - ref| / max |ref| per output row


def dev(x: np.ndarray, dtype=None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def kv_tensors(w: W.Workload):
    """q, k, v on the device in the workload's dtype (and paged pools when the workload is paged)."""
    dt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.dtype]
    q = dev(w.q, dt)
    if w.page_table is not None:
        k, v = dev(w.paged_pool(w.k), dt), dev(w.paged_pool(w.v), dt)
    else:
        k, v = dev(w.k, dt), dev(w.v, dt)
    return q, k, v


def gpu_select(probs: np.ndarray, top_p: float, *, seq_lens=None, capacity=None, page_table=None,
               page_size=0, emit_physical=False, probs_dev=None, split=True):
    """Run specattn_topp_select; returns dict of numpy results (+ device tensors).

    split: hand over the optional workspace, with which few long rows are split over many workgroups."""
    p = dev(probs) if probs_dev is None else probs_dev
    B, H, n = p.shape
    R = B * H
    cap = n if capacity is None else capacity
    idx = torch.full((R, cap), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    tau = torch.full((R,), -7.0, dtype=torch.float32, device="cuda")
    flags = torch.full((R,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    pt = None if page_table is None else dev(np.asarray(page_table, dtype=np.int32))
    args = sa.select_args(p, top_p, indices=idx, counts=counts, thresholds=tau, row_flags=flags,
                          seq_lens=sl, page_table=pt, page_size=page_size, emit_physical=emit_physical)
    need = sa.specattn_workspace_size(args, None) if split else 0
    ws = sa.alloc_workspace(need) if need else None
    sa.specattn_topp_select(args, ws)
    torch.cuda.synchronize()
    return dict(indices=idx.cpu().numpy(), counts=counts.cpu().numpy(), tau=tau.cpu().numpy(),
                flags=flags.cpu().numpy().astype(np.uint32), d_indices=idx, d_counts=counts,
                d_tau=tau, keep=(p, sl, pt), split=bool(need))


def compare_select(got: dict, ref: oracle.SelectResult, *, capacity=None, to_physical=None):
    """Bit-exact comparison off the rows the oracle flags as near-boundary.

    Returns (n_flagged, n_flagged_mismatched).  to_physical(row, positions) maps the oracle's
    logical positions to pool slots when the GPU emitted physical indices.
    """
    R = ref.counts.shape[0]
    flagged = mism = 0
    for r in range(R):
        want = ref.row_set(r)
        if to_physical is not None:
            want = to_physical(r, want)
        if ref.flags[r] & oracle.ROW_INVALID:
            assert got["flags"][r] & sa.ROW_INVALID, f"row {r}: invalid row not flagged"
            assert got["counts"][r] == 0
            continue
        assert not got["flags"][r] & sa.ROW_INVALID, f"row {r}: wrongly flagged invalid"
        n_got = int(got["counts"][r])
        cap = got["indices"].shape[1] if capacity is None else capacity
        same = (n_got == len(want) and got["tau"][r] == ref.tau[r] and
                np.array_equal(got["indices"][r, : min(n_got, cap)], want[:cap]))
        if ref.flags[r] & oracle.ROW_NEAR_BOUNDARY:
            flagged += 1
            mism += 0 if same else 1
            continue
        assert n_got == len(want), f"row {r}: count {n_got} != {len(want)}"
        assert got["tau"][r] == ref.tau[r], f"row {r}: tau {got['tau'][r]} != {ref.tau[r]}"
        assert np.array_equal(got["indices"][r, : min(n_got, cap)], want[:cap]), f"row {r}: index list differs"
        if n_got > cap:
            assert got["flags"][r] & sa.ROW_OVERFLOW
    return flagged, mism


def gpu_attention(q, k, v, indices, counts, *, page_table=None, page_size=0, physical=False,
                  n_max=None, want_lse=True):
    """Run specattn_sparse_decode_attn on device tensors; returns (out, lse) numpy."""
    B, H_q, T, d = q.shape
    out = torch.full((B, H_q, T, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H_q, T), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    args = sa.attn_args(q, k, v, out=out, indices=indices, counts=counts, lse=lse,
                        page_table=page_table, page_size=page_size, indices_are_physical=physical,
                        n_max=n_max)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, args))
    args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(args)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (None if lse is None else lse.cpu().numpy())


def oracle_attention(w: W.Workload, mask: np.ndarray, which=None):
    """Oracle output for the workload's logical q/k/v under mask [B,H_kv,n]."""
    if w.dtype == "bf16":
        qb, kb, vb = (W.round_to_bf16_bits(a).reshape(a.shape) for a in (w.q, w.k, w.v))
        return oracle.masked_attention(qb, kb, vb, mask, bf16=True, lens=w.seq_lens, which=which)
    if w.dtype == "f16":
        qb, kb, vb = (a.astype(np.float16).view(np.uint16) for a in (w.q, w.k, w.v))
        return oracle.masked_attention(qb, kb, vb, mask, f16=True, lens=w.seq_lens, which=which)
    return oracle.masked_attention(w.q, w.k, w.v, mask, lens=w.seq_lens, which=which)


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over output rows of max|got-ref| / max|ref| (rows with ref == 0 compare absolutely)."""
    g = got.reshape(-1, got.shape[-1]).astype(np.float64)
    r = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    scale = np.abs(r).max(axis=1)
    err = np.abs(g - r).max(axis=1)
    scale = np.where(scale > 0, scale, 1.0)
    return float((err / scale).max())
