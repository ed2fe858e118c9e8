"""The entry points allocate nothing and never synchronise, so a caller can record them in a HIP graph.
Each replay (with eager work and synchronisations in between) must reproduce the eager result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("path", ["unfused", "fused"])
def test_graph_replays_match_eager(path):
    w = W.llama8b_layer(seed=31, n=8192, top_p=0.95)
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    B, H, n = probs.shape
    R = B * H
    idx = torch.zeros((R, n), dtype=torch.int32, device="cuda")
    counts = torch.zeros((R,), dtype=torch.int32, device="cuda")
    tau = torch.zeros((R,), dtype=torch.float32, device="cuda")
    out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
    lse = torch.zeros(q.shape[:3], dtype=torch.float32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=idx if path == "unfused" else None, counts=counts, thresholds=tau)
    att = sa.attn_args(q, k, v, out=out, lse=lse, indices=idx, counts=counts)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(sel if path == "fused" else None, att))
    att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()

    def run():
        if path == "unfused":
            sa.specattn_topp_select(sel)
            sa.specattn_sparse_decode_attn(att)
        else:
            sa.specattn_fused(sel, att)

    def clear():
        for t in (idx, counts, tau, out, lse):
            t.zero_()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run()                                   # first call outside the capture (one-time kernel attributes)
        side.synchronize()
        eager = (out.cpu().numpy().copy(), lse.cpu().numpy().copy(), counts.cpu().numpy().copy())
        graph = torch.cuda.CUDAGraph()
        clear()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()

    ref = oracle.topp_select(w.probs.reshape(R, n), w.top_p)
    o_ref, _ = oracle_attention(w, ref.mask().reshape(B, H, n))
    assert row_rel_err(eager[0], o_ref) <= TOL["bf16"]
    for replay in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(counts.cpu().numpy(), eager[2]), f"replay {replay}: counts differ"
        assert row_rel_err(out.cpu().numpy(), eager[0]) <= 1e-5, f"replay {replay}: output differs from eager"
        assert np.abs(lse.cpu().numpy() - eager[1]).max() <= 1e-5
        # eager work of the program's own between the replays
        run()
        torch.cuda.synchronize()
        assert row_rel_err(out.cpu().numpy(), eager[0]) <= 1e-5
