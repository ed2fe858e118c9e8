"""Attention with the verifier's new tokens behind the cache (query t also attends to new tokens 0..t),
against the oracle; sparse, dense, paged and fused calls."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, kv_tensors, row_rel_err

pytestmark = pytest.mark.gpu


def new_tokens(w, seed):
    rng = np.random.default_rng(seed)
    shape = (w.B, w.H_kv, w.T, w.d)
    k_new = rng.standard_normal(shape, dtype=np.float32)
    v_new = rng.standard_normal(shape, dtype=np.float32)
    if w.dtype == "bf16":
        k_new, v_new = (W.bf16_bits_to_f32(W.round_to_bf16_bits(a)).reshape(shape) for a in (k_new, v_new))
    return k_new, v_new


def oracle_tail(w, mask, k_new, v_new):
    if w.dtype == "bf16":
        bits = lambda a: W.round_to_bf16_bits(a).reshape(a.shape)
        return oracle.masked_attention(bits(w.q), bits(w.k), bits(w.v), mask, bf16=True, lens=w.seq_lens,
                                       k_new=bits(k_new), v_new=bits(v_new))
    return oracle.masked_attention(w.q, w.k, w.v, mask, lens=w.seq_lens, k_new=k_new, v_new=v_new)


def run(w, k_new, v_new, *, mode, seq_lens=None, page_table=None):
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    q, k, v = kv_tensors(w)
    kn, vn = dev(k_new, dt), dev(v_new, dt)
    probs = dev(w.probs)
    B, H, n = probs.shape
    R = B * H
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    pt = None if page_table is None else dev(np.asarray(page_table, dtype=np.int32))
    ps = W.PAGE_SIZE if pt is not None else 0
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.zeros((R, n), dtype=torch.int32, device="cuda")
    counts = torch.zeros((R,), dtype=torch.int32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=idx if mode == "sparse" else None, counts=counts, seq_lens=sl)
    if mode == "dense":
        att = sa.attn_args(q, k, v, out=out, lse=lse, seq_lens=sl, page_table=pt, page_size=ps, n_max=n,
                           k_new=kn, v_new=vn)
    else:
        att = sa.attn_args(q, k, v, out=out, lse=lse, indices=idx, counts=counts, page_table=pt, page_size=ps,
                           n_max=n, k_new=kn, v_new=vn)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(sel if mode == "fused" else None, att))
    att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()
    if mode == "sparse":
        sa.specattn_topp_select(sel)
        sa.specattn_sparse_decode_attn(att)
    elif mode == "dense":
        sa.specattn_sparse_decode_attn(att)
    else:
        sa.specattn_fused(sel, att)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def reference(w, k_new, v_new, mode):
    B, H, n = w.probs.shape
    if mode == "dense":
        mask = np.zeros((B, H, n), dtype=bool)
        lens = w.row_lens().reshape(B, H)
        for b in range(B):
            for h in range(H):
                mask[b, h, :lens[b, h]] = True
    else:
        mask = oracle.topp_select(w.probs.reshape(B * H, n), w.top_p, lens=w.row_lens()).mask().reshape(B, H, n)
    return oracle_tail(w, mask, k_new, v_new)


@pytest.mark.parametrize("mode", ["sparse", "dense"])
def test_tiny_fp32_with_new_tokens(mode):
    w = W.tiny_f32(seed=21)
    k_new, v_new = new_tokens(w, 22)
    out, lse = run(w, k_new, v_new, mode=mode)
    o_ref, l_ref = reference(w, k_new, v_new, mode)
    assert row_rel_err(out, o_ref) <= TOL["f32"]
    assert np.abs(lse - l_ref).max() <= 1e-4


@pytest.mark.parametrize("mode", ["sparse", "dense", "fused"])
@pytest.mark.parametrize("n", [700, 8192])
def test_bf16_layer_with_new_tokens(mode, n):
    w = W.llama8b_layer(seed=23 + n, B=2, n=n, top_p=0.95)
    k_new, v_new = new_tokens(w, 24)
    out, lse = run(w, k_new, v_new, mode=mode)
    o_ref, l_ref = reference(w, k_new, v_new, mode)
    assert row_rel_err(out, o_ref) <= TOL["bf16"]
    assert np.abs(lse - l_ref).max() <= 1e-3


def test_many_rows_each_owned_by_one_workgroup():
    # more rows than workgroups: rows are finished by a single workgroup, yet still pick up the new tokens
    w = W.llama8b_layer(seed=29, B=80, n=256, top_p=0.9)
    k_new, v_new = new_tokens(w, 30)
    out, _ = run(w, k_new, v_new, mode="sparse")
    o_ref, _ = reference(w, k_new, v_new, "sparse")
    assert row_rel_err(out, o_ref) <= TOL["bf16"]


def test_empty_cache_attends_to_new_tokens_only():
    w = W.llama8b_layer(seed=31, B=3, n=512, top_p=0.9)
    lens = np.array([512, 0, 100], dtype=np.int32)
    w.seq_lens = lens
    w.probs[1] = 0.0
    w.probs[2, :, 100:] = 0.0
    k_new, v_new = new_tokens(w, 32)
    for mode in ("sparse", "dense"):
        out, lse = run(w, k_new, v_new, mode=mode, seq_lens=lens)
        o_ref, l_ref = reference(w, k_new, v_new, mode)
        assert row_rel_err(out, o_ref) <= TOL["bf16"]
        assert np.all(np.isfinite(lse))
        # query 0 of the empty sequence sees new token 0 only
        G = w.H_q // w.H_kv
        for hq in range(w.H_q):
            np.testing.assert_allclose(out[1, hq, 0], v_new[1, hq // G, 0], rtol=0, atol=1e-6)


def test_paged_with_new_tokens():
    w = W.ragged_paged(seed=33, B=5, len_lo=50, len_hi=3000)
    k_new, v_new = new_tokens(w, 34)
    for mode in ("sparse", "dense"):
        out, _ = run(w, k_new, v_new, mode=mode, seq_lens=w.seq_lens, page_table=w.page_table)
        o_ref, _ = reference(w, k_new, v_new, mode)
        assert row_rel_err(out, o_ref) <= TOL["bf16"]


@pytest.mark.parametrize("mode", ["sparse", "fused"])
def test_eight_query_heads_per_kv_head(mode):
    # 40 query rows per kv head: the matrix-core kernel runs the heads in two shares; the new tokens join in the merge
    w = W.llama8b_layer(seed=61, B=2, n=3000, top_p=0.9, H_q=64, H_kv=8)
    k_new, v_new = new_tokens(w, 62)
    out, lse = run(w, k_new, v_new, mode=mode)
    o_ref, l_ref = reference(w, k_new, v_new, mode)
    assert row_rel_err(out, o_ref) <= TOL["bf16"]
    assert np.abs(lse - l_ref).max() <= 1e-3
