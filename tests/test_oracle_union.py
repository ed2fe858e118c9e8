"""Pins for the oracle's union over draft steps and draft heads (Algorithm 2 as a whole; CPU only)."""
import numpy as np

import oracle


def _numpy_nucleus(row, p):
    """Textbook route written separately: argsort + cumsum; keeps ties at the threshold."""
    row = row.astype(np.float64)
    order = np.argsort(-row, kind="stable")
    cs = np.cumsum(row[order])
    kk = int(np.searchsorted(cs, float(np.float32(p)) * cs[-1], side="left"))
    return set(np.nonzero(row >= row[order[kk]])[0].tolist())


def test_hand_worked_union():
    # step 1 concentrates on position 0, step 2 on positions 3 and 2: p = 0.6
    #   step 1: 0.7 >= 0.6                      -> {0}
    #   step 2: 0.5 < 0.6, 0.5 + 0.3 >= 0.6     -> {2, 3}
    probs = np.array([[[[0.7, 0.1, 0.1, 0.1],
                        [0.1, 0.1, 0.3, 0.5]]]], dtype=np.float32)          # [B=1, H_d=1, S=2, n=4]
    res = oracle.topp_select_union(probs, 0.6, H_kv=1)
    assert res.counts[0] == 3 and list(res.row_set(0)) == [0, 2, 3]
    # two draft heads of one kv head, one step each: same union
    res2 = oracle.topp_select_union(probs.reshape(1, 2, 1, 4), 0.6, H_kv=1)
    assert list(res2.row_set(0)) == [0, 2, 3]
    # the same two heads feeding two kv heads: no union across kv heads
    res3 = oracle.topp_select_union(probs.reshape(1, 2, 1, 4), 0.6, H_kv=2)
    assert list(res3.row_set(0)) == [0] and list(res3.row_set(1)) == [2, 3]


def test_single_member_equals_plain_selection():
    rng = np.random.default_rng(0)
    probs = rng.dirichlet(np.full(300, 0.3), size=(2, 4)).astype(np.float32)     # [2, 4, 300]
    plain = oracle.topp_select(probs.reshape(8, 300), 0.9)
    uni = oracle.topp_select_union(probs.reshape(2, 4, 1, 300), 0.9, H_kv=4)
    for r in range(8):
        assert np.array_equal(plain.row_set(r), uni.row_set(r))
        assert plain.flags[r] == uni.flags[r]


def test_union_against_separate_numpy_route_with_lengths_and_gqa():
    rng = np.random.default_rng(1)
    B, H_d, S, n, H_kv = 3, 4, 3, 257, 2
    probs = rng.dirichlet(np.full(n, 0.2), size=(B, H_d, S)).astype(np.float32)
    lens = np.array([257, 100, 1], dtype=np.int32)
    for b in range(B):
        probs[b, :, :, lens[b]:] = 0.0
    res = oracle.topp_select_union(probs, 0.85, H_kv=H_kv, lens=lens)
    for b in range(B):
        for h in range(H_kv):
            r = b * H_kv + h
            if res.flags[r] & oracle.ROW_NEAR_BOUNDARY:
                continue
            want = set()
            for hd in (2 * h, 2 * h + 1):
                for s in range(S):
                    want |= _numpy_nucleus(probs[b, hd, s, :lens[b]], 0.85)
            assert sorted(want) == list(res.row_set(r))
            assert list(res.row_set(r)) == sorted(set(res.row_set(r)))        # ascending, no repeats


def test_union_contains_every_member_and_is_order_invariant():
    rng = np.random.default_rng(2)
    probs = rng.dirichlet(np.full(128, 0.5), size=(1, 2, 4)).astype(np.float32)
    res = oracle.topp_select_union(probs, 0.9, H_kv=1)
    for m in range(8):
        assert set(res.members.row_set(m)) <= set(res.row_set(0))
    flipped = probs[:, ::-1, ::-1].copy()
    res_f = oracle.topp_select_union(flipped, 0.9, H_kv=1)
    assert np.array_equal(res.row_set(0), res_f.row_set(0))


def test_invalid_members_are_skipped_and_all_invalid_row_is_flagged():
    probs = np.zeros((1, 2, 2, 8), dtype=np.float32)
    probs[0, 0, 0] = [0.5, 0.5, 0, 0, 0, 0, 0, 0]
    probs[0, 0, 1, 3] = np.nan                       # invalid member: contributes nothing
    res = oracle.topp_select_union(probs, 0.9, H_kv=2)
    assert list(res.row_set(0)) == [0, 1] and not res.flags[0] & oracle.ROW_INVALID
    assert res.counts[1] == 0 and res.flags[1] & oracle.ROW_INVALID       # head 1: all rows are zero
