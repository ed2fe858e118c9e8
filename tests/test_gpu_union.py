"""specattn_topp_select_union (Algorithm 2 as a whole: per-step top-p, then the union over steps and draft
heads) against the oracle: lists bit-exact wherever no member row sits within 1e-6 of its boundary."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, dev, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


def gpu_union(probs, top_p, H_kv, *, seq_lens=None, capacity=None, page_table=None, emit_physical=False):
    p = dev(probs)
    B, H_d, S, n = p.shape
    R = B * H_kv
    cap = n if capacity is None else capacity
    idx = torch.full((R, cap), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    flags = torch.full((R,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    mt = torch.full((B * H_d * S,), -7.0, dtype=torch.float32, device="cuda")
    mc = torch.full((B * H_d * S,), -7, dtype=torch.int32, device="cuda")
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    pt = None if page_table is None else dev(np.asarray(page_table, dtype=np.int32))
    a = sa.union_args(p, top_p, H_kv, indices=idx, counts=counts, row_flags=flags, seq_lens=sl,
                      member_thresholds=mt, member_counts=mc, page_table=pt, page_size=W.PAGE_SIZE if pt is not None else 0,
                      emit_physical=emit_physical)
    ws = sa.alloc_workspace(sa.specattn_union_workspace_size(a))
    sa.specattn_topp_select_union(a, ws)
    torch.cuda.synchronize()
    return dict(indices=idx.cpu().numpy(), counts=counts.cpu().numpy(), flags=flags.cpu().numpy().astype(np.uint32),
                tau=mt.cpu().numpy(), mcounts=mc.cpu().numpy(), d_indices=idx, d_counts=counts)


def compare(got, ref, *, capacity=None, to_physical=None):
    R = ref.counts.shape[0]
    flagged = mism = 0
    for r in range(R):
        want = ref.row_set(r)
        if to_physical is not None:
            want = to_physical(r, want)
        if ref.flags[r] & oracle.ROW_INVALID:
            assert got["flags"][r] & sa.ROW_INVALID and got["counts"][r] == 0
            continue
        assert not got["flags"][r] & sa.ROW_INVALID
        n_got = int(got["counts"][r])
        cap = got["indices"].shape[1] if capacity is None else capacity
        same = n_got == len(want) and np.array_equal(got["indices"][r, : min(n_got, cap)], want[:cap])
        if ref.flags[r] & oracle.ROW_NEAR_BOUNDARY:
            flagged += 1
            mism += 0 if same else 1
            continue
        assert n_got == len(want), f"row {r}: count {n_got} != {len(want)}"
        assert np.array_equal(got["indices"][r, : min(n_got, cap)], want[:cap]), f"row {r}: list differs"
        if n_got > cap:
            assert got["flags"][r] & sa.ROW_OVERFLOW
    # member thresholds: bit-exact off the flagged member rows
    mem = ref.members
    ok = (mem.flags & (oracle.ROW_NEAR_BOUNDARY | oracle.ROW_INVALID)) == 0
    assert np.array_equal(got["tau"][ok], mem.tau[ok])
    assert np.array_equal(got["mcounts"][ok], mem.counts[ok])
    return flagged, mism


@pytest.mark.parametrize("shape", [dict(B=1, H_d=1, S=1, n=1000, H_kv=1), dict(B=2, H_d=8, S=4, n=5000, H_kv=2),
                                   dict(B=1, H_d=4, S=3, n=4096, H_kv=4), dict(B=3, H_d=2, S=5, n=4097, H_kv=1),
                                   dict(B=1, H_d=2, S=2, n=70000, H_kv=2)])
def test_union_matches_oracle(shape):
    rng = np.random.default_rng(shape["n"] + shape["S"])
    probs = W.draft_step_probs(rng, shape["B"], shape["H_d"], shape["S"], shape["n"])
    got = gpu_union(probs, 0.9, shape["H_kv"])
    ref = oracle.topp_select_union(probs, 0.9, shape["H_kv"])
    flagged, mism = compare(got, ref)
    assert mism == 0, f"{mism} of {flagged} near-boundary rows differ"
    # the union is larger than any member's set and smaller than their sum
    assert (ref.counts >= ref.members.counts.reshape(ref.counts.shape[0], -1).max(axis=1)).all()


def test_ragged_lengths_invalid_members_and_capacity():
    rng = np.random.default_rng(5)
    lens = np.array([3000, 0, 17, 2048], dtype=np.int32)
    probs = W.draft_step_probs(rng, 4, 4, 3, 3000, lens=lens)
    probs[0, 1, 2, 5] = np.nan                        # one invalid member row: skipped
    probs[3, 2:, :, :] = 0.0                          # kv head 1 of sequence 3: every member row is zero
    got = gpu_union(probs, 0.95, 2, seq_lens=lens, capacity=600)
    ref = oracle.topp_select_union(probs, 0.95, 2, lens=lens)
    flagged, mism = compare(got, ref, capacity=600)
    assert mism == 0
    assert got["flags"][2] & sa.ROW_INVALID and got["flags"][3] & sa.ROW_INVALID       # empty sequence
    assert got["flags"][7] & sa.ROW_INVALID and not got["flags"][6] & sa.ROW_INVALID
    assert (got["flags"][(got["counts"] > 600)] & sa.ROW_OVERFLOW).all() and (got["counts"] > 600).any()


def test_paged_physical_output():
    w = W.ragged_paged(seed=9, B=4, len_lo=100, len_hi=6000, with_kv=False)
    rng = np.random.default_rng(10)
    probs = W.draft_step_probs(rng, 4, 8, 2, w.n, lens=w.seq_lens)
    got = gpu_union(probs, 0.9, 8, seq_lens=w.seq_lens, page_table=w.page_table, emit_physical=True)
    ref = oracle.topp_select_union(probs, 0.9, 8, lens=w.seq_lens)
    to_phys = lambda r, pos: w.page_table[r // 8, pos // W.PAGE_SIZE] * W.PAGE_SIZE + pos % W.PAGE_SIZE
    flagged, mism = compare(got, ref, to_physical=to_phys)
    assert mism == 0


def test_union_feeds_sparse_attention():
    w = W.llama8b_layer(seed=41, B=2, n=6000, top_p=0.9)
    rng = np.random.default_rng(42)
    probs = W.draft_step_probs(rng, 2, 16, 4, 6000)            # 16 draft heads -> 8 kv heads, 4 steps
    got = gpu_union(probs, 0.9, 8)
    ref = oracle.topp_select_union(probs, 0.9, 8)
    q, k, v = kv_tensors(w)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    a = sa.attn_args(q, k, v, out=out, indices=got["d_indices"], counts=got["d_counts"])
    ws = sa.alloc_workspace(sa.specattn_workspace_size(None, a))
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    sa.specattn_sparse_decode_attn(a)
    torch.cuda.synchronize()
    o_ref, _ = oracle_attention(w, ref.mask().reshape(2, 8, 6000))
    assert row_rel_err(out.cpu().numpy(), o_ref) <= TOL["bf16"]
