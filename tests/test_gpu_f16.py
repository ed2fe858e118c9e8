"""IEEE half K/V/Q through every attention route (the paper's own models run in fp16): list, fused, dense,
new tokens, paged, large GQA groups on the matrix-core kernel; d = 64 on the portable one."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def bits(a):
    return a.astype(np.float16).view(np.uint16)


def run(w, *, mode, k_new=None, v_new=None, paged=False):
    q, k, v = kv_tensors(w)
    assert q.dtype == torch.float16
    probs = dev(w.probs)
    B, H, n = probs.shape
    R = B * H
    sl = None if w.seq_lens is None else dev(np.asarray(w.seq_lens, dtype=np.int32))
    pt = dev(w.page_table) if paged else None
    ps = W.PAGE_SIZE if paged else 0
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.zeros((R, n), dtype=torch.int32, device="cuda")
    counts = torch.zeros((R,), dtype=torch.int32, device="cuda")
    kn = None if k_new is None else dev(k_new, torch.float16)
    vn = None if v_new is None else dev(v_new, torch.float16)
    sel = sa.select_args(probs, w.top_p, indices=idx if mode == "sparse" else None, counts=counts, seq_lens=sl)
    if mode == "dense":
        att = sa.attn_args(q, k, v, out=out, lse=lse, seq_lens=sl, page_table=pt, page_size=ps, n_max=n, k_new=kn, v_new=vn)
    else:
        att = sa.attn_args(q, k, v, out=out, lse=lse, indices=idx, counts=counts, page_table=pt, page_size=ps, n_max=n,
                           k_new=kn, v_new=vn)
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


def reference(w, mode, k_new=None, v_new=None):
    B, H, n = w.probs.shape
    lens = w.row_lens()
    if mode == "dense":
        mask = np.zeros((B * H, n), dtype=bool)
        for r in range(B * H):
            mask[r, :lens[r]] = True
    else:
        mask = oracle.topp_select(w.probs.reshape(B * H, n), w.top_p, lens=lens).mask()
    kw = {} if k_new is None else dict(k_new=bits(k_new), v_new=bits(v_new))
    return oracle.masked_attention(bits(w.q), bits(w.k), bits(w.v), mask.reshape(B, H, n), f16=True, lens=w.seq_lens, **kw)


@pytest.mark.parametrize("mode", ["sparse", "fused", "dense"])
@pytest.mark.parametrize("shape", [dict(), dict(H_q=8, H_kv=8, T=5), dict(H_q=64, H_kv=8, T=5)])
def test_half_layer(mode, shape):
    w = W.llama8b_layer(seed=71, B=2, n=5000, top_p=0.9, dtype="f16", **shape)
    out, lse = run(w, mode=mode)
    o_ref, l_ref = reference(w, mode)
    assert row_rel_err(out, o_ref) <= TOL["f16"]
    assert np.abs(lse - l_ref).max() <= 1e-3


def test_half_with_new_tokens_and_large_values():
    w = W.llama8b_layer(seed=72, B=2, n=3000, top_p=0.95, dtype="f16")
    w.v *= 300.0                                   # values near the top of the half range survive exactly
    w.v = w.v.astype(np.float16).astype(np.float32)
    rng = np.random.default_rng(73)
    k_new = rng.standard_normal((2, 8, 5, 128), dtype=np.float32).astype(np.float16).astype(np.float32)
    v_new = (300.0 * rng.standard_normal((2, 8, 5, 128), dtype=np.float32)).astype(np.float16).astype(np.float32)
    out, lse = run(w, mode="sparse", k_new=k_new, v_new=v_new)
    o_ref, l_ref = reference(w, "sparse", k_new, v_new)
    assert row_rel_err(out, o_ref) <= TOL["f16"]


def test_half_d64_on_the_portable_kernel():
    w = W.llama8b_layer(seed=74, B=2, n=1500, top_p=0.9, H_q=8, H_kv=2, T=5, d=64, dtype="f16")
    out, lse = run(w, mode="sparse")
    o_ref, l_ref = reference(w, "sparse")
    assert row_rel_err(out, o_ref) <= TOL["f16"]
