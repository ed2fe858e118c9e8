"""GPU parity: specattn_sparse_decode_attn (HIP, through the C ABI) against the oracle's masked
dense attention.  Tolerance: max |out - ref| / max |ref| per output row <= 2e-3 (bf16 inputs,
fp32 accumulation) or 1e-5 (fp32)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W
from helpers import TOL, dev, gpu_attention, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def _lists_from_mask(mask):
    """mask [B,H,n] -> (indices [B*H, n] int32 ascending, counts [B*H])."""
    B, H, n = mask.shape
    idx = np.zeros((B * H, n), dtype=np.int32)
    cnt = np.zeros(B * H, dtype=np.int32)
    for r in range(B * H):
        pos = np.nonzero(mask.reshape(B * H, n)[r])[0]
        idx[r, : len(pos)] = pos
        cnt[r] = len(pos)
    return idx, cnt


def _oracle_selection_mask(w):
    res = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p, w.row_lens())
    return res.mask().reshape(w.B, w.H_kv, w.n)


def _run_and_compare(w, mask, *, paged_mode=None, check_lse=True):
    idx, cnt = _lists_from_mask(mask)
    q, k, v = kv_tensors(w)
    kw = {}
    if w.page_table is not None:
        if paged_mode == "physical":
            for r in range(idx.shape[0]):
                b = r // w.H_kv
                p = idx[r, : cnt[r]]
                idx[r, : cnt[r]] = w.page_table[b, p // W.PAGE_SIZE] * W.PAGE_SIZE + p % W.PAGE_SIZE
            kw = dict(page_size=W.PAGE_SIZE, physical=True, n_max=w.n)
        else:
            kw = dict(page_table=dev(w.page_table), page_size=W.PAGE_SIZE, n_max=w.n)
    out, lse = gpu_attention(q, k, v, dev(idx), dev(cnt), **kw)
    ref, ref_lse = oracle_attention(w, mask)
    err = row_rel_err(out, ref)
    print(f"{w.name} B={w.B} n={w.n} dtype={w.dtype}: row-relative error {err:.3e}")
    assert np.isfinite(out).all()
    assert err <= TOL[w.dtype]
    if check_lse:
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(lse), np.isneginf(ref_lse))
        if fin.any():
            assert np.abs(lse[fin] - ref_lse[fin]).max() <= (2e-3 if w.dtype == "bf16" else 2e-5)
    return out, ref


def test_tiny_f32_workload():
    w = W.tiny_f32()
    _run_and_compare(w, _oracle_selection_mask(w))


def test_llama_layer_8k_bf16():
    w = W.llama8b_layer(seed=1)
    _run_and_compare(w, _oracle_selection_mask(w))


def test_batch_of_32k_rows_bf16():
    w = W.llama8b_layer(seed=3, B=2, n=32768, top_p=0.9)
    mask = _oracle_selection_mask(w)
    idx, cnt = _lists_from_mask(mask)
    q, k, v = kv_tensors(w)
    out, _ = gpu_attention(q, k, v, dev(idx), dev(cnt))
    rng = np.random.default_rng(0)
    which = [(int(rng.integers(w.B)), int(rng.integers(w.H_q)), int(rng.integers(w.T))) for _ in range(48)]
    ref, _ = oracle_attention(w, mask, which=which)
    got = np.stack([out[b, h, t] for b, h, t in which])
    assert row_rel_err(got, ref) <= TOL["bf16"]


def test_everything_selected_is_dense_attention():
    w = W.llama8b_layer(seed=4, n=1500)
    _run_and_compare(w, np.ones((w.B, w.H_kv, w.n), dtype=np.uint8))
    w = W.tiny_f32(seed=2, n=700)
    _run_and_compare(w, np.ones((w.B, w.H_kv, w.n), dtype=np.uint8))


@pytest.mark.parametrize("count", [0, 1, 2, 31, 32, 33, 255, 256, 257, 1000])
def test_ragged_list_lengths(count):
    w = W.llama8b_layer(seed=10 + count, n=2048)
    rng = np.random.default_rng(count)
    mask = np.zeros((w.B, w.H_kv, w.n), dtype=np.uint8)
    for h in range(w.H_kv):
        c = max(0, count - h) if h % 2 else count          # neighbouring rows differ in length
        mask[0, h, rng.choice(w.n, size=c, replace=False)] = 1
    out, ref = _run_and_compare(w, mask)
    if count == 0:
        assert (out[0, :4] == 0).all()


@pytest.mark.parametrize("shape", [
    dict(H_q=8, H_kv=8, T=1, d=128), dict(H_q=16, H_kv=2, T=8, d=128), dict(H_q=8, H_kv=2, T=5, d=64),
    dict(H_q=4, H_kv=4, T=3, d=64, dtype="f32"), dict(H_q=8, H_kv=4, T=5, d=128, dtype="f32"),
    # query rows per kv head at and around the matrix-core kernel's tile sizes (16 and 32)
    dict(H_q=8, H_kv=2, T=8, d=128), dict(H_q=4, H_kv=2, T=8, d=128), dict(H_q=6, H_kv=2, T=7, d=128),
    dict(H_q=2, H_kv=2, T=5, d=128), dict(H_q=34, H_kv=2, T=1, d=128), dict(H_q=22, H_kv=2, T=3, d=128),
    # more than 32 query rows per kv head: the matrix-core kernel takes the heads in equal shares
    dict(H_q=64, H_kv=8, T=5, d=128), dict(H_q=32, H_kv=2, T=8, d=128), dict(H_q=14, H_kv=2, T=5, d=128),
])
def test_other_shapes_and_dtypes(shape):
    w = W.llama8b_layer(seed=6, B=2, n=1300, **shape)
    _run_and_compare(w, _oracle_selection_mask(w))


def test_more_rows_than_one_launch_holds():
    # 2048 rows: the matrix-core variant runs them as two launches over consecutive sequences (1536 + 512 rows)
    w = W.llama8b_layer(seed=12, B=256, n=256, H_q=16, H_kv=8, T=2, top_p=0.7)
    _run_and_compare(w, _oracle_selection_mask(w))


@pytest.mark.parametrize("B", [9, 65, 88, 192, 193])
def test_row_counts_around_the_table_sizes(B):
    # 72, 520, 704, 1536 and 1544 rows: one wave's scan, one, two and three rounds of the workgroup-wide cost prefix,
    # and one row group past a full launch
    w = W.llama8b_layer(seed=13, B=B, n=200, H_q=16, H_kv=8, T=2, top_p=0.8)
    _run_and_compare(w, _oracle_selection_mask(w))


def test_one_selected_position_returns_its_value_row():
    w = W.llama8b_layer(seed=7, n=512)
    mask = np.zeros((w.B, w.H_kv, w.n), dtype=np.uint8)
    mask[:, :, 300] = 1
    out, _ = _run_and_compare(w, mask)
    for hq in range(w.H_q):
        assert np.array_equal(out[0, hq], np.broadcast_to(w.v[0, hq // w.G, 300], out[0, hq].shape))


@pytest.mark.parametrize("mode", ["table", "physical"])
def test_paged_ragged_batch(mode):
    w = W.ragged_paged(seed=2, B=5, len_lo=100, len_hi=6000)
    _run_and_compare(w, _oracle_selection_mask(w), paged_mode=mode)


def test_counts_above_capacity_are_clamped():
    w = W.llama8b_layer(seed=8, n=1024)
    mask = np.zeros((w.B, w.H_kv, w.n), dtype=np.uint8)
    mask[:, :, :200] = 1
    idx, cnt = _lists_from_mask(mask)
    q, k, v = kv_tensors(w)
    out, _ = gpu_attention(q, k, v, dev(idx[:, :200].copy()), dev(cnt + 5000))
    ref, _ = oracle_attention(w, mask)
    assert row_rel_err(out, ref) <= TOL["bf16"]


def test_select_then_attend_end_to_end():
    """Both library calls chained on the device, against oracle selection + oracle attention."""
    from helpers import gpu_select
    w = W.llama8b_layer(seed=9, B=2, n=8192)
    sel = gpu_select(w.probs, w.top_p)
    q, k, v = kv_tensors(w)
    out, _ = gpu_attention(q, k, v, sel["d_indices"], sel["d_counts"])
    ref, _ = oracle_attention(w, _oracle_selection_mask(w))
    assert row_rel_err(out, ref) <= TOL["bf16"]


def test_outputs_are_bit_identical_run_to_run():
    """Tiles go to waves and workgroups by the counts alone and the partials of a row are merged in workgroup order:
    repeated calls agree bit for bit (out and lse), in rows owned by one workgroup as in rows split over several."""
    for w in (W.llama8b_layer(seed=11, n=4096), W.llama8b_layer(seed=12, B=4, n=16384, top_p=0.9)):
        idx, cnt = _lists_from_mask(_oracle_selection_mask(w))
        q, k, v = kv_tensors(w)
        a, a_lse = gpu_attention(q, k, v, dev(idx), dev(cnt))
        for _ in range(3):
            b, b_lse = gpu_attention(q, k, v, dev(idx), dev(cnt))
            assert np.array_equal(a, b) and np.array_equal(a_lse, b_lse)
        ref, _ = oracle_attention(w, _oracle_selection_mask(w))
        assert row_rel_err(a, ref) <= TOL["bf16"]


def test_few_rows_and_table_lookups_agree():
    """Up to 64 rows a workgroup finds its rows with one ballot, beyond that by searching the cost prefix
    table.  A ninth, empty sequence (rows without kept positions cost nothing, so the shares stay the same)
    sends the same eight sequences down the other way: same outputs up to the summation order."""
    w = W.llama8b_layer(seed=21, B=8, n=4096)
    idx, cnt = _lists_from_mask(_oracle_selection_mask(w))
    q, k, v = kv_tensors(w)
    a, a_lse = gpu_attention(q, k, v, dev(idx), dev(cnt))
    pad = lambda t: torch.cat([t, torch.zeros_like(t[:1])], dim=0)
    idx9 = np.concatenate([idx, np.zeros((w.H_kv, idx.shape[1]), dtype=np.int32)])
    cnt9 = np.concatenate([cnt, np.zeros(w.H_kv, dtype=np.int32)])
    b, b_lse = gpu_attention(pad(q), pad(k), pad(v), dev(idx9), dev(cnt9))
    assert row_rel_err(b[:8], a) <= 1e-5
    assert np.abs(b_lse[:8] - a_lse).max() <= 1e-5
    assert (b[8] == 0).all() and np.isneginf(b_lse[8]).all()
    ref, _ = oracle_attention(w, _oracle_selection_mask(w))
    assert row_rel_err(a, ref) <= TOL["bf16"]
