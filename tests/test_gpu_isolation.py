"""No hidden shared state and no stray writes: concurrent calls on two streams with their own workspaces give the
results of the serial calls, and nothing outside the documented outputs is touched."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import dev, kv_tensors

pytestmark = pytest.mark.gpu

GUARD = 64


def _guarded(shape, dtype, fill):
    """A tensor of `shape` carved out of a larger buffer whose margins hold a known pattern."""
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    return buf, buf[GUARD:GUARD + n].view(shape)


def _margins_intact(buf, fill):
    b = buf.cpu()
    return bool((b[:GUARD] == fill).all() and (b[-GUARD:] == fill).all())


def test_two_streams_with_own_workspaces():
    ws_, outs, args = [], [], []
    works = [W.llama8b_layer(seed=51, B=2, n=6000, top_p=0.9), W.llama8b_layer(seed=52, B=3, n=4000, top_p=0.95)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for w in works:
        q, k, v = kv_tensors(w)
        probs = dev(w.probs)
        B, H, n = probs.shape
        idx = torch.zeros((B * H, n), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((B * H,), dtype=torch.int32, device="cuda")
        out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
        sel = sa.select_args(probs, w.top_p, indices=idx, counts=cnt)
        att = sa.attn_args(q, k, v, out=out, indices=idx, counts=cnt)
        ws = sa.alloc_workspace(sa.specattn_workspace_size(None, att))
        att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()
        ws_.append((ws, q, k, v, probs, idx, cnt))
        outs.append(out)
        args.append((sel, att))
    serial = []
    for (sel, att), out in zip(args, outs):
        sa.specattn_topp_select(sel)
        sa.specattn_sparse_decode_attn(att)
        torch.cuda.synchronize()
        serial.append(out.cpu().numpy().copy())
        out.zero_()
    torch.cuda.synchronize()
    for rep in range(5):
        for (sel, att), st in zip(args, streams):
            sa.specattn_topp_select(sel, stream=st)
            sa.specattn_sparse_decode_attn(att, stream=st)
    torch.cuda.synchronize()
    for out, ref in zip(outs, serial):
        got = out.cpu().numpy()
        scale = np.abs(ref).max(axis=-1, keepdims=True)
        assert (np.abs(got - ref) / scale).max() <= 1e-5


def test_nothing_outside_the_outputs_is_written():
    w = W.llama8b_layer(seed=53, B=2, n=5000, top_p=0.9)
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    B, H, n = probs.shape
    R = B * H
    cap = 300                                              # well below the kept counts: lists are truncated
    ibuf, idx = _guarded((R, cap), torch.int32, -77)
    cbuf, cnt = _guarded((R,), torch.int32, -77)
    tbuf, tau = _guarded((R,), torch.float32, -77.0)
    fbuf, flg = _guarded((R,), torch.int32, -77)
    obuf, out = _guarded(tuple(q.shape), torch.float32, -77.0)
    lbuf, lse = _guarded(tuple(q.shape[:3]), torch.float32, -77.0)
    sel = sa.select_args(probs, w.top_p, indices=idx, counts=cnt, thresholds=tau, row_flags=flg)
    att = sa.attn_args(q, k, v, out=out, lse=lse, indices=idx, counts=cnt)
    need = sa.specattn_workspace_size(None, att)
    wbuf = torch.full((need + 2 * 256,), 0x5A, dtype=torch.uint8, device="cuda")
    att.workspace, att.workspace_bytes = wbuf.data_ptr() + 256, need
    sa.specattn_topp_select(sel)
    sa.specattn_sparse_decode_attn(att)
    torch.cuda.synchronize()
    assert (cnt.cpu().numpy() > cap).all() and (flg.cpu().numpy() & sa.ROW_OVERFLOW).all()
    for buf, fill in ((ibuf, -77), (cbuf, -77), (tbuf, -77.0), (fbuf, -77), (obuf, -77.0), (lbuf, -77.0)):
        assert _margins_intact(buf, fill)
    wb = wbuf.cpu()
    assert bool((wb[:256] == 0x5A).all() and (wb[-256:] == 0x5A).all())
    # the truncated lists are the first `cap` entries of the full ones
    ref = oracle.topp_select(w.probs.reshape(R, n), w.top_p)
    got = idx.cpu().numpy()
    for r in range(R):
        if not ref.flags[r] & oracle.ROW_NEAR_BOUNDARY:
            assert np.array_equal(got[r], ref.row_set(r)[:cap])
    # union, chunk and bisection modes write inside their lists as well
    ubuf, uidx = _guarded((R, cap), torch.int32, -77)
    rng = np.random.default_rng(54)
    ps = dev(W.draft_step_probs(rng, B, H, 3, n))
    ua = sa.union_args(ps, 0.9, H, indices=uidx, counts=cnt)
    sa.specattn_topp_select_union(ua, sa.alloc_workspace(sa.specattn_union_workspace_size(ua)))
    bbuf, bidx = _guarded((R, cap), torch.int32, -77)
    ba = sa.select_args(probs, 0.9, indices=bidx, counts=cnt, bisect_iters=10)
    sa.specattn_topp_select(ba, sa.alloc_workspace(sa.specattn_workspace_size(ba, None)))
    kbuf, kidx = _guarded((R, 40), torch.int32, -77)
    ka = sa.select_args(probs, 0.9, indices=kidx, counts=cnt, chunk_size=16)
    sa.specattn_topp_select(ka, sa.alloc_workspace(sa.specattn_workspace_size(ka, None)))
    torch.cuda.synchronize()
    for buf in (ubuf, bbuf, kbuf, cbuf):
        assert _margins_intact(buf, -77)


@pytest.mark.parametrize("H_q", [32, 64, 128])
@pytest.mark.parametrize("mode", ["list", "fused"])
def test_workspace_is_never_exceeded_whatever_the_group_size(H_q, mode):
    """Every workgroup may leave a partial in the workspace, and groups of more than 32 query rows per kv head run
    as several launches over it: a wide margin behind the workspace of the size the query reports stays untouched."""
    w = W.llama8b_layer(seed=55, B=2, n=6000, top_p=0.9, H_q=H_q, H_kv=8)
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    B, H, n = probs.shape
    idx = torch.zeros((B * H, n), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((B * H,), dtype=torch.int32, device="cuda")
    out = torch.full(tuple(q.shape), float("nan"), dtype=torch.float32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=idx if mode == "list" else None, counts=cnt)
    att = sa.attn_args(q, k, v, out=out, indices=idx, counts=cnt) if mode == "list" else sa.attn_args(q, k, v, out=out)
    need = sa.specattn_workspace_size(sel if mode == "fused" else None, att)
    margin = 8 << 20
    wbuf = torch.full((256 + need + margin,), 0x5A, dtype=torch.uint8, device="cuda")
    att.workspace, att.workspace_bytes = wbuf.data_ptr() + 256, need
    if mode == "list":
        sa.specattn_topp_select(sel)
        sa.specattn_sparse_decode_attn(att)
    else:
        sa.specattn_fused(sel, att)
    torch.cuda.synchronize()
    assert bool((wbuf[:256] == 0x5A).all().item()) and bool((wbuf[256 + need:] == 0x5A).all().item())
    assert bool(torch.isfinite(out).all().item())
    # a workspace one byte short is refused before anything is launched
    att.workspace_bytes = need - 1
    with pytest.raises(sa.SpecAttnError):
        if mode == "list":
            sa.specattn_sparse_decode_attn(att)
        else:
            sa.specattn_fused(sel, att)


def test_layer_mapping_writes_only_its_outputs():
    ad, av = W.layer_attention_maps(seed=56, m=7, n=11, rows=9, L=300)
    sbuf, S = _guarded((7, 11), torch.float64, -77.0)
    fbuf, f = _guarded((11,), torch.int32, -77)
    tbuf, tot = _guarded((1,), torch.float64, -77.0)
    lib = sa.load()
    n1 = int(lib.specattn_layer_similarity_workspace_size(7, 11, 9, 300))
    n2 = int(lib.specattn_layer_map_workspace_size(7, 11))
    w1 = torch.full((n1 + 512,), 0x5A, dtype=torch.uint8, device="cuda")
    w2 = torch.full((n2 + 512,), 0x5A, dtype=torch.uint8, device="cuda")
    sa.specattn_layer_similarity(dev(ad), dev(av), S, workspace=w1[256:256 + n1])
    sa.specattn_layer_map(S, f, tot, workspace=w2[256:256 + n2])
    torch.cuda.synchronize()
    for buf, fill in ((sbuf, -77.0), (fbuf, -77), (tbuf, -77.0)):
        assert _margins_intact(buf, fill)
    for wb, nn in ((w1, n1), (w2, n2)):
        assert bool((wb[:256] == 0x5A).all().item()) and bool((wb[256 + nn:] == 0x5A).all().item())
    f_ref, v_ref = oracle.layer_map(oracle.layer_similarity_fast(ad, av))
    assert np.array_equal(f.cpu().numpy(), f_ref) and abs(tot.item() - v_ref) <= 1e-9 * abs(v_ref)
