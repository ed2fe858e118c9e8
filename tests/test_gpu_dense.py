"""Dense calls of the attention entry point (no index list: every position below the sequence length),
against the oracle's masked attention with an all-true mask."""
import numpy as np
import pytest
import torch

from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def dense_call(w, q, k, v, *, seq_lens=None, page_table=None, page_size=0, n_max=None):
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    pt = None if page_table is None else dev(np.asarray(page_table, dtype=np.int32))
    a = sa.attn_args(q, k, v, out=out, lse=lse, seq_lens=sl, page_table=pt, page_size=page_size, n_max=n_max)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(a)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def full_mask(w):
    B, H, n = w.probs.shape
    m = np.zeros((B, H, n), dtype=bool)
    lens = w.row_lens().reshape(B, H)
    for b in range(B):
        for h in range(H):
            m[b, h, :lens[b, h]] = True
    return m


def test_tiny_fp32_dense():
    w = W.tiny_f32(seed=3)
    q, k, v = kv_tensors(w)
    out, lse = dense_call(w, q, k, v)
    o_ref, l_ref = oracle_attention(w, full_mask(w))
    assert row_rel_err(out, o_ref) <= TOL["f32"]
    assert np.abs(lse - l_ref).max() <= 1e-4


@pytest.mark.parametrize("n", [1, 31, 32, 33, 4096, 8192 + 17])
def test_bf16_dense_lengths(n):
    w = W.llama8b_layer(seed=100 + n, n=n, top_p=0.9)
    q, k, v = kv_tensors(w)
    out, lse = dense_call(w, q, k, v)
    o_ref, l_ref = oracle_attention(w, full_mask(w))
    assert row_rel_err(out, o_ref) <= TOL["bf16"]
    assert np.abs(lse - l_ref).max() <= 1e-3


def test_bf16_dense_ragged_with_empty_sequence():
    w = W.llama8b_layer(seed=7, B=4, n=3000, top_p=0.9)
    lens = np.array([3000, 0, 1234, 17], dtype=np.int32)
    w.seq_lens = lens
    q, k, v = kv_tensors(w)
    out, lse = dense_call(w, q, k, v, seq_lens=lens)
    o_ref, l_ref = oracle_attention(w, full_mask(w))
    assert row_rel_err(out, o_ref) <= TOL["bf16"]
    assert np.all(out[1] == 0.0) and np.all(np.isneginf(lse[1]))
    ok = np.isfinite(l_ref)
    assert np.abs(lse[ok] - l_ref[ok]).max() <= 1e-3


def test_bf16_dense_paged():
    w = W.ragged_paged(seed=5, B=6, len_lo=100, len_hi=5000)
    q, k, v = kv_tensors(w)
    out, lse = dense_call(w, q, k, v, seq_lens=w.seq_lens, page_table=w.page_table, page_size=W.PAGE_SIZE,
                          n_max=w.probs.shape[2])
    o_ref, l_ref = oracle_attention(w, full_mask(w))
    assert row_rel_err(out, o_ref) <= TOL["bf16"]
