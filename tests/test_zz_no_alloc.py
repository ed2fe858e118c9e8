"""The entry point that allocates nothing: specattn_sparse_decode_attn_static keeps its split partials in a
buffer that is part of the library image.  Its outputs must equal those of specattn_sparse_decode_attn (the
same kernels on a caller workspace) and stay within the oracle's tolerance, on two calls in a row that share
the buffer, the second on a smaller input."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, gpu_select, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def _both_entry_points(w):
    ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p)
    got = gpu_select(w.probs, w.top_p)
    q, k, v = kv_tensors(w)
    B, H_q, T, d = q.shape
    outs, lses = [], []
    for static in (False, True):
        out = torch.full((B, H_q, T, d), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((B, H_q, T), float("nan"), dtype=torch.float32, device="cuda")
        args = sa.attn_args(q, k, v, out=out, indices=got["d_indices"], counts=got["d_counts"], lse=lse)
        if static:
            before = torch.cuda.memory_allocated()
            sa.specattn_sparse_decode_attn_static(args)            # workspace stays NULL
            assert torch.cuda.memory_allocated() == before
        else:
            ws = sa.alloc_workspace(sa.specattn_workspace_size(None, args))
            args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel()
            sa.specattn_sparse_decode_attn(args)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        lses.append(lse.cpu().numpy())
    want, want_lse = oracle_attention(w, ref.mask().reshape(w.B, w.H_kv, w.n))
    return outs, lses, want, want_lse


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    # the second call is smaller than the first, so it finds the first call's partials in the shared buffer
    for w in (W.llama8b_layer(seed=41, n=8192, top_p=0.95), W.llama8b_layer(seed=42, n=2048, top_p=0.9)):
        outs, lses, want, want_lse = _both_entry_points(w)
        assert not np.isnan(outs[1]).any() and not np.isnan(lses[1]).any()
        # the two entry points run the same kernels: only the summation order of a launch may differ
        assert row_rel_err(outs[1], outs[0]) <= 1e-5
        assert np.abs(lses[1] - lses[0]).max() <= 1e-5
        assert row_rel_err(outs[1], want) <= TOL[w.dtype]
        assert np.abs(lses[1] - want_lse).max() <= 1e-3


def test_static_scratch_takes_large_batches_in_smaller_launches():
    # 1600 rows: the workspace call takes them as 1536 + 64 rows, the built-in buffer holds launches of 512 rows
    w = W.llama8b_layer(seed=43, B=200, n=200, H_q=16, H_kv=8, T=2, top_p=0.8)
    outs, lses, want, want_lse = _both_entry_points(w)
    assert row_rel_err(outs[1], outs[0]) <= 1e-5
    assert row_rel_err(outs[1], want) <= TOL[w.dtype]
    assert np.abs(lses[1] - want_lse).max() <= 1e-3


def test_static_scratch_fp32_route_and_size_limit():
    w = W.tiny_f32()
    outs, lses, want, _ = _both_entry_points(w)
    assert row_rel_err(outs[1], outs[0]) <= 1e-6
    assert row_rel_err(outs[1], want) <= TOL["f32"]
    # a call whose partials cannot fit the built-in buffer is refused before anything is launched
    q = torch.zeros((512, 32, 5, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((512, 8, 64, 128), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((512 * 8, 64), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((512 * 8,), dtype=torch.int32, device="cuda")
    out = torch.zeros((512, 32, 5, 128), dtype=torch.float32, device="cuda")
    args = sa.attn_args(q, k, k, out=out, indices=idx, counts=cnt)
    assert sa.specattn_workspace_size(None, args) > (16 << 20)
    with pytest.raises(sa.SpecAttnError) as e:
        sa.specattn_sparse_decode_attn_static(args)
    assert e.value.status == sa.EWORKSPACE
