"""Chunk-granular selection (chunk masses, exact top-p over them) and attention over chunk lists, against the
oracle: chunk lists and thresholds bit-exact off the near-boundary rows, outputs within the attention tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, compare_select, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def gpu_select_chunks(probs, top_p, chunk, *, seq_lens=None, capacity=None):
    p = dev(probs)
    B, H, n = p.shape
    R = B * H
    nc = (n + chunk - 1) // chunk
    cap = nc if capacity is None else capacity
    idx = torch.full((R, cap), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    tau = torch.full((R,), -7.0, dtype=torch.float32, device="cuda")
    flags = torch.full((R,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    a = sa.select_args(p, top_p, indices=idx, counts=counts, thresholds=tau, row_flags=flags, seq_lens=sl,
                       chunk_size=chunk)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(a, None))
    sa.specattn_topp_select(a, ws)
    torch.cuda.synchronize()
    return dict(indices=idx.cpu().numpy(), counts=counts.cpu().numpy(), tau=tau.cpu().numpy(),
                flags=flags.cpu().numpy().astype(np.uint32), d_indices=idx, d_counts=counts, d_lens=sl)


@pytest.mark.parametrize("chunk", [2, 16, 64])
@pytest.mark.parametrize("n", [16, 1000, 4096, 40000])
def test_chunk_lists_match_oracle(chunk, n):
    rng = np.random.default_rng(n + chunk)
    probs = W.draft_probs(rng, 6, n).reshape(2, 3, n)
    got = gpu_select_chunks(probs, 0.9, chunk)
    ref = oracle.topp_select_chunks(probs.reshape(6, n), 0.9, chunk)
    flagged, mism = compare_select(got, ref)
    assert mism == 0


def test_ragged_lengths_partial_chunks_and_invalid_rows():
    rng = np.random.default_rng(3)
    lens = np.array([5000, 0, 4999, 17, 16, 1], dtype=np.int32)
    probs = W.draft_probs(rng, 12, 5000, lens=np.repeat(lens, 2)).reshape(6, 2, 5000)
    probs[0, 1, 77] = -1.0                     # hides inside a positive chunk mass unless checked per entry
    got = gpu_select_chunks(probs, 0.95, 16, seq_lens=lens)
    ref = oracle.topp_select_chunks(probs.reshape(12, 5000), 0.95, 16, lens=np.repeat(lens, 2))
    flagged, mism = compare_select(got, ref)
    assert mism == 0
    assert got["flags"][1] & sa.ROW_INVALID and got["flags"][2] & sa.ROW_INVALID


@pytest.mark.parametrize("paged", [False, True])
def test_attention_over_chunk_lists(paged):
    if paged:
        w = W.ragged_paged(seed=11, B=5, len_lo=40, len_hi=6000)
        lens = w.seq_lens
    else:
        w = W.llama8b_layer(seed=12, B=3, n=5000, top_p=0.9)
        lens = np.array([5000, 4097, 33], dtype=np.int32)        # partial last chunks (the recency band keeps them)
        w.seq_lens = lens
        for b in range(3):
            w.probs[b, :, lens[b]:] = 0.0
    B, H, n = w.probs.shape
    got = gpu_select_chunks(w.probs, w.top_p, 16, seq_lens=lens)
    ref = oracle.topp_select_chunks(w.probs.reshape(B * H, n), w.top_p, 16, lens=np.repeat(lens, H))
    flagged, mism = compare_select(got, ref)
    assert mism == 0
    mask = oracle.chunk_token_mask(ref, 16, n, np.repeat(lens, H)).reshape(B, H, n)
    q, k, v = kv_tensors(w)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    pt = dev(w.page_table) if paged else None
    a = sa.attn_args(q, k, v, out=out, lse=lse, indices=got["d_indices"], counts=got["d_counts"], seq_lens=got["d_lens"],
                     page_table=pt, page_size=W.PAGE_SIZE if paged else 0, n_max=n, chunk_size=16)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(a)
    torch.cuda.synchronize()
    o_ref, l_ref = oracle_attention(w, mask)
    assert row_rel_err(out.cpu().numpy(), o_ref) <= TOL["bf16"]
    assert np.abs(lse.cpu().numpy() - l_ref).max() <= 1e-3


def test_tiny_fp32_chunks_through_the_portable_kernel():
    w = W.tiny_f32(seed=13)
    B, H, n = w.probs.shape
    got = gpu_select_chunks(w.probs, 0.9, 16)
    ref = oracle.topp_select_chunks(w.probs.reshape(B * H, n), 0.9, 16)
    assert compare_select(got, ref)[1] == 0
    mask = oracle.chunk_token_mask(ref, 16, n).reshape(B, H, n)
    q, k, v = kv_tensors(w)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    a = sa.attn_args(q, k, v, out=out, indices=got["d_indices"], counts=got["d_counts"], chunk_size=16)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(a)
    torch.cuda.synchronize()
    o_ref, _ = oracle_attention(w, mask)
    assert row_rel_err(out.cpu().numpy(), o_ref) <= TOL["f32"]
