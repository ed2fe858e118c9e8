"""The optional second output copy in the input dtype equals the fp32 output rounded to nearest even, on every
route that finishes a row (single-owner rows, merged rows, empty rows, the portable kernel)."""
import numpy as np
import pytest
import torch

from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import dev, kv_tensors

pytestmark = pytest.mark.gpu


def _run(w, *, new_tokens=False):
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    B, H, n = probs.shape
    idx = torch.zeros((B * H, n), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((B * H,), dtype=torch.int32, device="cuda")
    sa.specattn_topp_select(sa.select_args(probs, w.top_p, indices=idx, counts=cnt))
    cnt[0] = 0                                              # an empty row: zeros in both copies
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    low = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    kn = vn = None
    if new_tokens:
        g = torch.Generator(device="cuda"); g.manual_seed(3)
        kn = torch.randn((B, H, w.T, w.d), device="cuda", generator=g).to(q.dtype)
        vn = torch.randn((B, H, w.T, w.d), device="cuda", generator=g).to(q.dtype)
    a = sa.attn_args(q, k, v, out=out, indices=idx, counts=cnt, out_lowp=low, k_new=kn, v_new=vn)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(a)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    assert torch.equal(low, out.to(q.dtype)), "low-precision copy is not the rounded fp32 output"
    if not new_tokens:
        G = w.H_q // w.H_kv
        assert (low[0, :G] == 0).all()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_rows_shared_by_several_workgroups(dtype):
    kw = dict(d=64, H_q=8, H_kv=4) if dtype == "f32" else {}
    _run(W.llama8b_layer(seed=81, B=2, n=6000, top_p=0.9, dtype=dtype, **kw))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_rows_owned_by_one_workgroup_and_new_tokens(dtype):
    _run(W.llama8b_layer(seed=82, B=80, n=256, top_p=0.9, dtype=dtype))
    _run(W.llama8b_layer(seed=83, B=2, n=3000, top_p=0.9, dtype=dtype), new_tokens=True)
