"""GPU parity of specattn_fused (selection + attention without an index list in HBM) against
oracle selection followed by oracle masked attention."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W
from helpers import TOL, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def _fused(w, *, reuse=False, give_state=False, want_lse=True):
    """Run specattn_fused on workload w; returns (out, lse, counts, tau)."""
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    R = w.B * w.H_kv
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    sl = None if w.seq_lens is None else dev(w.seq_lens.astype(np.int32))
    pt = None if w.page_table is None else dev(w.page_table)
    nblk = (w.n + sa.SEL_BLOCK - 1) // sa.SEL_BLOCK
    tau = torch.zeros((R,), dtype=torch.float32, device="cuda") if (give_state or reuse) else None
    bc = torch.full((R, nblk), -1, dtype=torch.int32, device="cuda") if (give_state or reuse) else None
    km = torch.full((R, nblk * 32), -1, dtype=torch.int32, device="cuda") if (give_state or reuse) else None
    out = torch.full((w.B, w.H_q, w.T, w.d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.B, w.H_q, w.T), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    if reuse:      # the threshold phase as a separate (batchable) call that writes no index list
        s0 = sa.select_args(probs, w.top_p, indices=None, counts=counts, thresholds=tau, seq_lens=sl,
                            block_counts=bc, kept_mask=km)
        sa.specattn_topp_select(s0)
    sel = sa.select_args(probs, w.top_p, indices=None, counts=counts, thresholds=tau, seq_lens=sl,
                         block_counts=bc, kept_mask=km, reuse_selection=reuse)
    kw = dict(page_table=pt, page_size=W.PAGE_SIZE, n_max=w.n) if pt is not None else dict(n_max=w.n)
    att = sa.attn_args(q, k, v, out=out, lse=lse, seq_lens=sl, **kw)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(sel, att))
    att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_fused(sel, att)
    torch.cuda.synchronize()
    return (out.cpu().numpy(), None if lse is None else lse.cpu().numpy(), counts.cpu().numpy(),
            None if tau is None else tau.cpu().numpy())


def test_kept_mask_and_block_counts_equal_the_oracle_set():
    """The selection state the fused call works from: one bit per position and kept counts per 1024 positions,
    bit for bit the oracle's kept set (off the rows the oracle flags as near the boundary)."""
    for w in (W.llama8b_layer(seed=8, B=2, n=5000, top_p=0.9), W.ragged_paged(seed=4, B=6, len_lo=50, len_hi=7000),
              W.llama8b_layer(seed=9, B=1, n=70001, H_q=8, H_kv=2, top_p=0.95)):
        probs = dev(w.probs)
        R = w.B * w.H_kv
        nblk = (w.n + sa.SEL_BLOCK - 1) // sa.SEL_BLOCK
        counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
        bc = torch.full((R, nblk), -1, dtype=torch.int32, device="cuda")
        km = torch.full((R, nblk * 32), -1, dtype=torch.int32, device="cuda")
        sl = None if w.seq_lens is None else dev(w.seq_lens.astype(np.int32))
        sa.specattn_topp_select(sa.select_args(probs, w.top_p, indices=None, counts=counts, seq_lens=sl,
                                               block_counts=bc, kept_mask=km))
        torch.cuda.synchronize()
        ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p, w.row_lens())
        want = np.zeros((R, nblk * 1024), dtype=np.uint8)
        want[:, :w.n] = ref.mask().reshape(R, w.n)
        got = np.unpackbits(km.cpu().numpy().view(np.uint8), axis=1, bitorder="little")
        clear = (ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0
        assert clear.any()
        assert np.array_equal(got[clear], want[clear])
        assert np.array_equal(bc.cpu().numpy()[clear], want.reshape(R, nblk, 1024).sum(axis=2)[clear])
        assert np.array_equal(counts.cpu().numpy()[clear], ref.counts[clear])


def _reference(w, which=None):
    ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p, w.row_lens())
    mask = ref.mask().reshape(w.B, w.H_kv, w.n)
    o, lse = oracle_attention(w, mask, which=which)
    return ref, o, lse


def _check_counts(counts, ref):
    clear = (ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0
    assert np.array_equal(counts[clear], ref.counts[clear])


@pytest.mark.parametrize("mode", ["one_call", "state_given", "reuse"])
def test_llama_layer_8k(mode):
    w = W.llama8b_layer(seed=1)
    out, lse, counts, tau = _fused(w, reuse=(mode == "reuse"), give_state=(mode == "state_given"))
    ref, o, l = _reference(w)
    _check_counts(counts, ref)
    assert row_rel_err(out, o) <= TOL["bf16"]
    assert np.abs(lse - l).max() <= 2e-3
    if tau is not None:
        clear = (ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0
        assert np.array_equal(tau[clear], ref.tau[clear])


def test_batch_of_32k_rows_sampled():
    w = W.llama8b_layer(seed=3, B=2, n=32768, top_p=0.9)
    out, _, counts, _ = _fused(w)
    rng = np.random.default_rng(1)
    which = [(int(rng.integers(w.B)), int(rng.integers(w.H_q)), int(rng.integers(w.T))) for _ in range(48)]
    ref, o, _ = _reference(w, which=which)
    _check_counts(counts, ref)
    got = np.stack([out[b, h, t] for b, h, t in which])
    assert row_rel_err(got, o) <= TOL["bf16"]


@pytest.mark.parametrize("n", [33, 1000, 1024, 1025, 5000, 70001])
def test_row_lengths(n):
    w = W.llama8b_layer(seed=20 + n % 7, B=2, n=n, H_q=8, H_kv=2, top_p=0.9)
    out, _, counts, _ = _fused(w)
    ref, o, _ = _reference(w)
    _check_counts(counts, ref)
    assert row_rel_err(out, o) <= TOL["bf16"]


def test_sparse_rows_whose_tiles_span_many_mask_words():
    """Kept positions far apart: the 32 positions of a tile lie in more than the 64 mask words fetched ahead
    (row 0: one kept position in about 130; row 1: two clusters 30000 positions apart; row 2: 3 kept positions;
    row 3 as drawn), so the on-chip decode takes further rounds over the following words."""
    w = W.llama8b_layer(seed=31, B=1, n=40000, H_q=8, H_kv=4, top_p=0.9)
    rng = np.random.default_rng(5)
    base = rng.random((3, w.n)).astype(np.float32) * 1e-9
    spikes = np.sort(rng.choice(w.n, size=300, replace=False))
    base[0, spikes] = 1.0 + rng.random(300).astype(np.float32)
    base[1, 100:140] = 1.0
    base[1, 30100:30140] = 1.0
    base[2, [5, 20000, 39999]] = 1.0
    w.probs[0, :3] = base
    out, lse, counts, _ = _fused(w)
    ref, o, l = _reference(w)
    _check_counts(counts, ref)
    assert 200 < counts[0] < 300 and counts[1] == 80 and counts[2] == 3      # (ties at the threshold are all kept)
    assert row_rel_err(out, o) <= TOL["bf16"]
    assert np.abs(lse - l).max() <= 2e-3


@pytest.mark.parametrize("B", [80, 200])
def test_many_rows_through_the_mask_source(B):
    # 640 rows (two rounds of the workgroup-wide cost prefix) and 1600 rows (1536 + 64: two launches)
    w = W.llama8b_layer(seed=33, B=B, n=300, H_q=16, H_kv=8, T=2, top_p=0.8)
    out, lse, counts, _ = _fused(w)
    ref, o, l = _reference(w)
    _check_counts(counts, ref)
    assert row_rel_err(out, o) <= TOL["bf16"]


def test_paged_ragged_batch_through_page_table():
    w = W.ragged_paged(seed=4, B=6, len_lo=50, len_hi=7000)
    out, lse, counts, _ = _fused(w)
    ref, o, l = _reference(w)
    _check_counts(counts, ref)
    assert row_rel_err(out, o) <= TOL["bf16"]


def test_invalid_and_empty_rows_give_zero_output():
    w = W.llama8b_layer(seed=5, n=3000, H_q=8, H_kv=4)
    w.probs[0, 1, 17] = np.nan
    w.probs[0, 2, :] = 0.0
    out, lse, counts, _ = _fused(w)
    ref, o, l = _reference(w)
    assert counts[1] == 0 and counts[2] == 0
    G = w.G
    assert (out[0, 1 * G:(2 + 1) * G] == 0).all()
    assert np.isneginf(lse[0, 1 * G:(2 + 1) * G]).all()
    assert row_rel_err(out, o) <= TOL["bf16"]


def test_top_p_one_selects_everything():
    w = W.llama8b_layer(seed=6, n=2100, top_p=1.0, H_q=8, H_kv=2)
    out, _, counts, _ = _fused(w)
    ref, o, _ = _reference(w)
    assert (counts == 2100).all()
    assert row_rel_err(out, o) <= TOL["bf16"]


def test_tiny_fp32_workload_through_the_fused_entry():
    """fp32, d = 64: the fused entry runs the selection into its workspace and attends over that list."""
    w = W.tiny_f32()
    out, lse, counts, _ = _fused(w)
    ref, o, l = _reference(w)
    _check_counts(counts, ref)
    assert row_rel_err(out, o) <= TOL["f32"]
    assert np.abs(lse - l).max() <= 1e-4
    with pytest.raises(sa.SpecAttnError) as e:          # the on-chip selection state does not exist on this route
        _fused(w, give_state=True)
    assert e.value.status == sa.EUNSUPPORTED


@pytest.mark.parametrize("chunk", [16, 64])
def test_chunk_granular_selection_through_the_fused_entry(chunk):
    """sel.chunk_size > 1: top-p over chunk masses, attention over every position of the kept chunks."""
    w = W.llama8b_layer(seed=13, B=2, n=5000, top_p=0.9)
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    R = w.B * w.H_kv
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    out = torch.full((w.B, w.H_q, w.T, w.d), float("nan"), dtype=torch.float32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=None, counts=counts, chunk_size=chunk)
    att = sa.attn_args(q, k, v, out=out, n_max=w.n)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(sel, att))
    att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_fused(sel, att)
    torch.cuda.synchronize()
    ref = oracle.topp_select_chunks(w.probs.reshape(-1, w.n), w.top_p, chunk)
    clear = (ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0
    assert np.array_equal(counts.cpu().numpy()[clear], ref.counts[clear])
    mask = oracle.chunk_token_mask(ref, chunk, w.n, np.full(R, w.n, dtype=np.int32)).reshape(w.B, w.H_kv, w.n)
    o, _ = oracle_attention(w, mask)
    assert row_rel_err(out.cpu().numpy(), o) <= TOL["bf16"]


def test_physical_indices_do_not_apply_to_the_fused_entry():
    w = W.ragged_paged(seed=4, B=2, len_lo=50, len_hi=900)
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    counts = torch.zeros((w.B * w.H_kv,), dtype=torch.int32, device="cuda")
    out = torch.zeros((w.B, w.H_q, w.T, w.d), dtype=torch.float32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=None, counts=counts, seq_lens=dev(w.seq_lens.astype(np.int32)))
    att = sa.attn_args(q, k, v, out=out, page_size=W.PAGE_SIZE, n_max=w.n, indices_are_physical=True)
    ws = sa.alloc_workspace(1 << 24)
    att.workspace, att.workspace_bytes = ws.data_ptr(), ws.numel()
    with pytest.raises(sa.SpecAttnError) as e:
        sa.specattn_fused(sel, att)
    assert e.value.status == sa.EUNSUPPORTED
