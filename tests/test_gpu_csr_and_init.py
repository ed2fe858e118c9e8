"""CSR form of the selection's lists (Section 3.5 hands the mask to the paper's attention kernel as CSR), the
optional device set-up call, and a first attention call recorded in a HIP graph."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import TOL, compare_select, dev, gpu_select, kv_tensors, oracle_attention, row_rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("capacity", [None, 300])
def test_csr_row_pointers_and_packed_entries(capacity):
    w = W.ragged_paged(seed=7, B=5, len_lo=40, len_hi=3000)
    lens = np.repeat(w.seq_lens, w.H_kv)
    ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p, lens)
    got = gpu_select(w.probs, w.top_p, seq_lens=w.seq_lens, capacity=capacity)
    compare_select(got, ref, capacity=capacity)
    R = ref.counts.size
    cap = w.n if capacity is None else capacity
    indptr = torch.full((R + 1,), -1, dtype=torch.int64, device="cuda")
    packed = torch.full((R * cap,), -1, dtype=torch.int32, device="cuda")
    sa.specattn_lists_to_csr(got["d_indices"], got["d_counts"], indptr, packed)
    torch.cuda.synchronize()
    clear = (ref.flags & oracle.ROW_NEAR_BOUNDARY) == 0
    lengths = np.minimum(np.where(clear, ref.counts, got["counts"]), cap)       # flagged rows: whatever the device kept
    want_ptr = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
    assert np.array_equal(indptr.cpu().numpy(), want_ptr)
    pk = packed.cpu().numpy()
    for r in range(R):
        if clear[r]:
            assert np.array_equal(pk[want_ptr[r]:want_ptr[r + 1]], ref.row_set(r)[:cap])
    assert (pk[want_ptr[-1]:] == -1).all()
    # row pointers alone (no entries wanted), with counts above the capacity clamped
    ind2 = torch.zeros((R + 1,), dtype=torch.int64, device="cuda")
    sa.specattn_lists_to_csr(None, got["d_counts"], ind2, None, capacity=7)
    torch.cuda.synchronize()
    assert np.array_equal(ind2.cpu().numpy(), np.concatenate([[0], np.cumsum(np.minimum(got["counts"], 7).astype(np.int64))]))


def test_many_rows_take_several_rounds_of_the_scan():
    R = 2500
    counts = torch.from_numpy(np.random.default_rng(3).integers(-2, 50, R).astype(np.int32)).cuda()
    indptr = torch.zeros((R + 1,), dtype=torch.int64, device="cuda")
    sa.specattn_lists_to_csr(None, counts, indptr, None, capacity=40)
    torch.cuda.synchronize()
    c = np.clip(counts.cpu().numpy(), 0, 40).astype(np.int64)
    assert np.array_equal(indptr.cpu().numpy(), np.concatenate([[0], np.cumsum(c)]))


def test_first_call_of_a_kernel_variant_inside_a_graph_capture():
    """specattn_init sets every kernel attribute up front, so a variant that has never run (fp16, pool-slot lists,
    one query tile) can make its first call under stream capture; the replays must reproduce an eager call."""
    sa.specattn_init()
    sa.specattn_init()                                   # any number of times
    w = W.ragged_paged(seed=9, B=3, len_lo=100, len_hi=2500, H_q=8, H_kv=4, T=2)
    w.dtype = "f16"
    ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p, np.repeat(w.seq_lens, w.H_kv))
    got = gpu_select(w.probs, w.top_p, seq_lens=w.seq_lens, page_table=w.page_table, page_size=W.PAGE_SIZE, emit_physical=True)
    q, k, v = kv_tensors(w)
    out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
    att = sa.attn_args(q, k, v, out=out, indices=got["d_indices"], counts=got["d_counts"], page_size=W.PAGE_SIZE,
                       n_max=w.n, indices_are_physical=True)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sa.specattn_sparse_decode_attn_static(att)   # nothing allocated, nothing set up under capture
    torch.cuda.synchronize()
    want, _ = oracle_attention(w, ref.mask().reshape(w.B, w.H_kv, w.n))
    for _ in range(2):
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert row_rel_err(out.cpu().numpy(), want) <= TOL["f16"]


def test_first_call_of_a_vector_alu_variant_inside_a_graph_capture():
    """The same for the kernels that take d = 64 (fp16 with d = 64 has not run before this test in a run of the whole suite)."""
    sa.specattn_init()
    w = W.tiny_f32(seed=3, n=700, B=2, H=4, T=3)
    w.dtype = "f16"
    ref = oracle.topp_select(w.probs.reshape(-1, w.n), w.top_p)
    got = gpu_select(w.probs, w.top_p)
    q, k, v = kv_tensors(w)
    out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
    att = sa.attn_args(q, k, v, out=out, indices=got["d_indices"], counts=got["d_counts"])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sa.specattn_sparse_decode_attn_static(att)
    torch.cuda.synchronize()
    want, _ = oracle_attention(w, ref.mask().reshape(w.B, w.H_kv, w.n))
    for _ in range(2):
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert row_rel_err(out.cpu().numpy(), want) <= TOL["f16"]
