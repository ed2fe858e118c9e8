"""GPU parity at the full sizes of the workload list, in the launch configuration bench.py times:
selection is compared on every row, attention on sampled output rows that the oracle computes one
by one (each sample is a 1-query, 1-kv-head problem cut out of the device tensors) and, for the headline
layer, on every output row."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W
from helpers import TOL, compare_select, dev, gpu_select, row_rel_err

pytestmark = pytest.mark.gpu


def _device_qkv(seed, B, H_q, H_kv, T, d, n_rows_kv, paged_pages=0):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    q = torch.randn((B, H_q, T, d), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    shape = (paged_pages, H_kv, W.PAGE_SIZE, d) if paged_pages else (B, H_kv, n_rows_kv, d)
    k = torch.randn(shape, generator=g, device="cuda", dtype=torch.bfloat16)
    v = torch.randn(shape, generator=g, device="cuda", dtype=torch.bfloat16)
    return q, k, v


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _sample_check(out, q, k_of, v_of, ref, H_kv, G, n, lens, samples):
    """out [B,H_q,T,d] (numpy); k_of(b, hk) -> [len, d] bf16 device tensor of logical rows."""
    worst = 0.0
    for (b, hq, t) in samples:
        hk = hq // G
        r = b * H_kv + hk
        L = int(lens[b])
        kk, vv = _bits(k_of(b, hk))[None, None], _bits(v_of(b, hk))[None, None]
        qq = _bits(q[b, hq, t])[None, None, None]
        mask = np.zeros((1, 1, L), dtype=np.uint8)
        mask[0, 0, ref.row_set(r)] = 1
        o, _ = oracle.masked_attention(qq, kk, vv, mask, bf16=True)
        worst = max(worst, row_rel_err(out[b, hq, t][None], o.reshape(1, -1)))
    return worst


def _attend(q, k, v, sel, *, fused_args=None, **kw):
    B, H_q, T, d = q.shape
    out = torch.full((B, H_q, T, d), float("nan"), dtype=torch.float32, device="cuda")
    if fused_args is None:
        a = sa.attn_args(q, k, v, out=out, indices=sel["d_indices"], counts=sel["d_counts"], **kw)
        ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
        a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
        sa.specattn_sparse_decode_attn(a)
    else:
        s = fused_args
        a = sa.attn_args(q, k, v, out=out, **kw)
        ws = sa.alloc_workspace(sa.specattn_workspace_size(s, a))
        a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
        sa.specattn_fused(s, a)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_headline_layer_b8_n32768_unfused_and_fused():
    B, H_q, H_kv, T, d, n, top_p = 8, 32, 8, 5, 128, 32768, 0.9
    w = W.llama8b_layer(seed=1000, B=B, n=n, top_p=top_p, with_kv=False)
    ref = oracle.topp_select(w.probs.reshape(-1, n), top_p)
    sel = gpu_select(w.probs, top_p)
    flagged, mism = compare_select(sel, ref)
    print(f"headline layer: kept fraction {sel['counts'].mean() / n:.4f}, flagged rows {flagged}, mismatched {mism}")
    assert mism == 0
    q, k, v = _device_qkv(7, B, H_q, H_kv, T, d, n)
    rng = np.random.default_rng(0)
    samples = [(int(rng.integers(B)), int(rng.integers(H_q)), int(rng.integers(T))) for _ in range(40)]
    lens = np.full(B, n)
    out = _attend(q, k, v, sel)
    assert np.isfinite(out).all()
    err = _sample_check(out, q, lambda b, h: k[b, h], lambda b, h: v[b, h], ref, H_kv, H_q // H_kv, n, lens, samples)
    probs_d = sel["keep"][0]
    counts = torch.zeros((B * H_kv,), dtype=torch.int32, device="cuda")
    s = sa.select_args(probs_d, top_p, indices=None, counts=counts)
    out_f = _attend(q, k, v, sel, fused_args=s, n_max=n)
    err_f = _sample_check(out_f, q, lambda b, h: k[b, h], lambda b, h: v[b, h], ref, H_kv, H_q // H_kv, n, lens, samples)
    print(f"headline layer: sampled row-relative error unfused {err:.2e}, fused {err_f:.2e}")
    assert err <= TOL["bf16"] and err_f <= TOL["bf16"]
    # every output row of the layer (1280 of them) against the oracle's masked dense attention over the whole layer
    mask = ref.mask().reshape(B, H_kv, n)
    o, _ = oracle.masked_attention(_bits(q), _bits(k), _bits(v), mask, bf16=True)
    err_all = row_rel_err(out, o)
    clear = np.repeat(((ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0).reshape(B, H_kv), H_q // H_kv, axis=1)   # per query head
    err_all_f = row_rel_err(out_f[clear], o[clear])
    print(f"headline layer: row-relative error over all {B * H_q * T} output rows unfused {err_all:.2e}, fused {err_all_f:.2e}")
    assert err_all <= TOL["bf16"] and err_all_f <= TOL["bf16"]


@pytest.mark.parametrize("clip", [None, 8.0])
def test_long_context_b4_n131072_top_p_sweep(clip):
    B, H_q, H_kv, T, d, n = 4, 32, 8, 5, 128, 131072
    w = W.long_context(seed=3, B=B, n=n, logit_clip=clip, with_kv=False)
    q, k, v = _device_qkv(11, B, H_q, H_kv, T, d, n)
    probs_d = dev(w.probs)
    rng = np.random.default_rng(1)
    for top_p in (0.8, 0.9, 0.95, 0.99):
        ref = oracle.topp_select(w.probs.reshape(-1, n), top_p)
        t0 = time.time()
        sel = gpu_select(None, top_p, probs_dev=probs_d)
        flagged, mism = compare_select(sel, ref)
        assert mism == 0
        samples = [(int(rng.integers(B)), int(rng.integers(H_q)), int(rng.integers(T))) for _ in range(6)]
        out = _attend(q, k, v, sel)
        err = _sample_check(out, q, lambda b, h: k[b, h], lambda b, h: v[b, h], ref, H_kv, H_q // H_kv, n,
                            np.full(B, n), samples)
        print(f"long context clip={clip} top_p={top_p}: kept fraction {sel['counts'].mean() / n:.5f} "
              f"(min {sel['counts'].min()}, max {sel['counts'].max()}), flagged {flagged}, sampled error {err:.2e}")
        assert err <= TOL["bf16"]


def test_ragged_paged_batch_b64():
    B, H_q, H_kv, T, d, top_p = 64, 32, 8, 5, 128, 0.95
    w = W.ragged_paged(seed=0, B=B, with_kv=False)
    n = w.n
    ref = oracle.topp_select(w.probs.reshape(-1, n), top_p, w.row_lens())
    pt = dev(w.page_table)
    sl = dev(w.seq_lens.astype(np.int32))
    q, kp, vp = _device_qkv(13, B, H_q, H_kv, T, d, 0, paged_pages=w.n_pool_pages)
    G = H_q // H_kv

    def logical(pool):
        def f(b, h):
            L = int(w.seq_lens[b])
            pages = torch.from_numpy(w.page_table[b, : (L + W.PAGE_SIZE - 1) // W.PAGE_SIZE].astype(np.int64)).cuda()
            return pool[pages, h].reshape(-1, d)[:L]
        return f

    rng = np.random.default_rng(2)
    samples = [(int(rng.integers(B)), int(rng.integers(H_q)), int(rng.integers(T))) for _ in range(24)]
    for mode in ("table", "physical", "fused"):
        if mode == "physical":
            sel = gpu_select(w.probs, top_p, seq_lens=w.seq_lens, page_table=w.page_table,
                             page_size=W.PAGE_SIZE, emit_physical=True)
            kw = dict(page_size=W.PAGE_SIZE, indices_are_physical=True, n_max=n)
        else:
            sel = gpu_select(w.probs, top_p, seq_lens=w.seq_lens)
            assert compare_select(sel, ref)[1] == 0
            kw = dict(page_table=pt, page_size=W.PAGE_SIZE, n_max=n)
        fused = None
        if mode == "fused":
            counts = torch.zeros((B * H_kv,), dtype=torch.int32, device="cuda")
            fused = sa.select_args(sel["keep"][0], top_p, indices=None, counts=counts, seq_lens=sl)
            kw["seq_lens"] = sl
        out = _attend(q, kp, vp, sel, fused_args=fused, **kw)
        assert np.isfinite(out).all()
        err = _sample_check(out, q, logical(kp), logical(vp), ref, H_kv, G, n, w.seq_lens, samples)
        print(f"ragged paged B=64 ({int(w.seq_lens.sum())} tokens, kept fraction "
              f"{ref.counts.sum() / w.row_lens().sum():.4f}) mode={mode}: sampled error {err:.2e}")
        assert err <= TOL["bf16"]
