"""specattn_check_lists: lists written by the selection pass; planted mistakes are counted."""
import numpy as np
import pytest
import torch

from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import dev, kv_tensors

pytestmark = pytest.mark.gpu


def _setup(w, *, paged=False, physical=False, chunk=0):
    q, k, v = kv_tensors(w)
    probs = dev(w.probs)
    B, H, n = probs.shape
    sl = None if w.seq_lens is None else dev(np.asarray(w.seq_lens, dtype=np.int32))
    pt = dev(w.page_table) if paged else None
    cap = n if not chunk else (n + chunk - 1) // chunk
    idx = torch.zeros((B * H, cap), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((B * H,), dtype=torch.int32, device="cuda")
    sel = sa.select_args(probs, w.top_p, indices=idx, counts=cnt, seq_lens=sl, page_table=pt,
                         page_size=W.PAGE_SIZE if paged else 0, emit_physical=physical, chunk_size=chunk)
    need = sa.specattn_workspace_size(sel, None)
    sa.specattn_topp_select(sel, sa.alloc_workspace(need) if need else None)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    att = sa.attn_args(q, k, v, out=out, indices=idx, counts=cnt, seq_lens=sl, page_table=pt,
                       page_size=W.PAGE_SIZE if paged else 0, n_max=n, indices_are_physical=physical, chunk_size=chunk)
    return att, idx, cnt, (q, k, v, probs, sl, pt, out)


def _bad(att, pool_slots=0):
    n_bad = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    sa.specattn_check_lists(att, n_bad, pool_slots)
    torch.cuda.synchronize()
    return int(n_bad.item())


def test_lists_from_the_selection_are_clean_and_planted_mistakes_are_counted():
    w = W.llama8b_layer(seed=91, B=2, n=4000, top_p=0.9)
    att, idx, cnt, keep = _setup(w)
    assert _bad(att) == 0
    idx[3, 10] = 4000                     # beyond the sequence
    idx[5, 7] = idx[5, 6]                 # a repeat
    idx[6, 0] = -1                        # negative
    cnt[9] = -2                           # a negative count
    # 4000 is out of range and also breaks the order of its successor; the repeat, the negative entry and the
    # negative count add one each
    assert _bad(att) == 5


def test_paged_physical_and_chunk_lists():
    w = W.ragged_paged(seed=92, B=4, len_lo=100, len_hi=3000)
    slots = w.n_pool_pages * W.PAGE_SIZE
    att, idx, cnt, keep = _setup(w, paged=True)
    assert _bad(att, slots) == 0
    keep[5][0, 0] = w.n_pool_pages        # page table entry of a listed position beyond the pool (position 0 is the sink)
    assert _bad(att, slots) >= 8          # every kv head of sequence 0 lists position 0
    att, idx, cnt, keep = _setup(w, paged=True, physical=True)
    assert _bad(att, slots) == 0
    idx[0, 0] = slots
    assert _bad(att, slots) == 1
    w2 = W.llama8b_layer(seed=93, B=2, n=4001, top_p=0.9)
    att, idx, cnt, keep = _setup(w2, chunk=16)
    assert _bad(att) == 0
    idx[1, 0] = 251                       # 4001 positions are 251 chunks: 0..250
    assert _bad(att) >= 1
