"""The paper-compatible mode of the selection (Algorithm 2 with a fixed number of halvings) against the
oracle: lists and thresholds bit-exact on every row none of whose comparisons was within 1e-6 of the target."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import binding as sa
from paper_2510_27641_amd import workloads as W

from helpers import compare_select, dev

pytestmark = pytest.mark.gpu


def gpu_bisect(probs, top_p, iters, *, seq_lens=None, capacity=None):
    p = dev(probs)
    B, H, n = p.shape
    R = B * H
    cap = n if capacity is None else capacity
    idx = torch.full((R, cap), -7, dtype=torch.int32, device="cuda")
    counts = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    tau = torch.full((R,), -7.0, dtype=torch.float32, device="cuda")
    flags = torch.full((R,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    a = sa.select_args(p, top_p, indices=idx, counts=counts, thresholds=tau, row_flags=flags, seq_lens=sl,
                       bisect_iters=iters)
    ws = sa.alloc_workspace(sa.specattn_workspace_size(a, None))
    sa.specattn_topp_select(a, ws)
    torch.cuda.synchronize()
    return dict(indices=idx.cpu().numpy(), counts=counts.cpu().numpy(), tau=tau.cpu().numpy(),
                flags=flags.cpu().numpy().astype(np.uint32))


@pytest.mark.parametrize("iters", [1, 10, 30])
@pytest.mark.parametrize("n", [7, 1000, 4096, 33000])
def test_matches_oracle(iters, n):
    rng = np.random.default_rng(n + iters)
    probs = W.draft_probs(rng, 6, n).reshape(2, 3, n)
    got = gpu_bisect(probs, 0.9, iters)
    ref = oracle.bisection_select(probs.reshape(6, n), 0.9, iters)
    flagged, mism = compare_select(got, ref)
    assert mism == 0


def test_ten_halvings_keep_everything_under_a_sink_where_the_exact_nucleus_is_small():
    # long-context rows with a literal Student-t draw: one position carries nearly all mass
    w = W.long_context(seed=2, B=1, n=131072, with_kv=False)
    B, H, n = w.probs.shape
    got = gpu_bisect(w.probs, 0.99, 10)
    ref = oracle.bisection_select(w.probs.reshape(B * H, n), 0.99, 10)
    flagged, mism = compare_select(got, ref)
    assert mism == 0
    exact = oracle.topp_select(w.probs.reshape(B * H, n), 0.99)
    assert (got["counts"] >= exact.counts).all()


def test_ragged_lengths_zeros_and_invalid_rows():
    rng = np.random.default_rng(4)
    lens = np.array([3000, 0, 2999, 5], dtype=np.int32)
    probs = W.draft_probs(rng, 8, 3000, lens=np.repeat(lens, 2)).reshape(4, 2, 3000)
    probs[0, 0, 100:200] = 0.0                   # zeros inside the row: kept only if theta_low stays 0
    probs[2, 1, 9] = np.inf
    for iters, p in ((10, 0.9), (3, 1.0)):
        got = gpu_bisect(probs, p, iters, seq_lens=lens, capacity=2500)
        ref = oracle.bisection_select(probs.reshape(8, 3000), p, iters, lens=np.repeat(lens, 2))
        flagged, mism = compare_select(got, ref, capacity=2500)
        assert mism == 0
        assert got["flags"][5] & sa.ROW_INVALID and got["flags"][2] & sa.ROW_INVALID
    # p = 1: the full mass is only reached at theta_low = 0, which keeps the zeros and nothing past the length
    assert got["counts"][0] == 3000 and got["counts"][6] == 5
