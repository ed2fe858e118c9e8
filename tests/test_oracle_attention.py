"""Pins for the oracle's masked attention (CPU only).

The oracle is compared with a library attention routine (torch's
scaled_dot_product_attention in fp64, with and without a boolean mask), with
special cases whose answer is known without any attention code, and with
identities that follow from Eq. 1-3 and Appendix A.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_27641_amd import workloads as W


def _rand(seed, B=2, H_q=8, H_kv=2, T=3, d=16, n=97):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H_q, T, d), dtype=np.float32)
    k = rng.standard_normal((B, H_kv, n, d), dtype=np.float32)
    v = rng.standard_normal((B, H_kv, n, d), dtype=np.float32)
    mask = (rng.random((B, H_kv, n)) < 0.3).astype(np.uint8)
    mask[..., 0] = 1
    return q, k, v, mask


def _sdpa(q, k, v, mask=None):
    G = q.shape[1] // k.shape[1]
    tq = torch.from_numpy(q).double()
    tk = torch.from_numpy(k).double().repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v).double().repeat_interleave(G, dim=1)
    am = None
    if mask is not None:
        am = torch.from_numpy(mask.astype(bool)).repeat_interleave(G, dim=1)[:, :, None, :]
        am = am.expand(-1, -1, q.shape[2], -1)
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=am).numpy()


def test_all_selected_equals_library_dense_attention():
    q, k, v, _ = _rand(0)
    ones = np.ones(k.shape[:3], dtype=np.uint8)
    o, _ = oracle.masked_attention(q, k, v, ones)
    np.testing.assert_allclose(o, _sdpa(q, k, v), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("shape", [dict(), dict(B=1, H_q=4, H_kv=4, T=5, d=64, n=130),
                                   dict(B=3, H_q=6, H_kv=3, T=1, d=8, n=33)])
def test_masked_equals_library_masked_attention(shape):
    q, k, v, mask = _rand(1, **shape)
    o, _ = oracle.masked_attention(q, k, v, mask)
    np.testing.assert_allclose(o, _sdpa(q, k, v, mask), rtol=1e-10, atol=1e-12)


def test_gqa_head_mapping_is_consecutive():
    # kv head 1 carries a constant V of 7: exactly the query heads 4..7 of 8 must see it
    q, k, v, _ = _rand(2, B=1, H_q=8, H_kv=2)
    v[:, 0] = -3.0
    v[:, 1] = 7.0
    ones = np.ones(k.shape[:3], dtype=np.uint8)
    o, _ = oracle.masked_attention(q, k, v, ones)
    np.testing.assert_allclose(o[0, :4], -3.0, rtol=1e-12)
    np.testing.assert_allclose(o[0, 4:], 7.0, rtol=1e-12)


def test_single_selected_position_returns_its_value_row():
    q, k, v, _ = _rand(3)
    mask = np.zeros(k.shape[:3], dtype=np.uint8)
    mask[:, :, 41] = 1
    o, lse = oracle.masked_attention(q, k, v, mask)
    G = q.shape[1] // k.shape[1]
    for hq in range(q.shape[1]):
        np.testing.assert_array_equal(o[:, hq], np.broadcast_to(
            v[:, hq // G, 41][:, None, :].astype(np.float64), o[:, hq].shape))
    # and the log-sum-exp is the one kept score
    s = np.einsum("bhtd,bhd->bht", q.astype(np.float64),
                  np.repeat(k[:, :, 41].astype(np.float64), G, axis=1)) / np.sqrt(q.shape[-1])
    np.testing.assert_allclose(lse, s, rtol=1e-12, atol=1e-12)


def test_constant_keys_give_mean_of_selected_values():
    q, k, v, mask = _rand(4)
    k[:] = k[:, :, :1]          # every key equal: uniform weights over the kept positions
    o, _ = oracle.masked_attention(q, k, v, mask)
    G = q.shape[1] // k.shape[1]
    for b in range(q.shape[0]):
        for hq in range(q.shape[1]):
            sel = mask[b, hq // G].astype(bool)
            want = v[b, hq // G][sel].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(o[b, hq], np.broadcast_to(want, o[b, hq].shape), rtol=1e-11,
                                       atol=1e-13)


def test_lse_merge_of_two_halves_equals_whole():
    q, k, v, mask = _rand(5)
    m1, m2 = mask.copy(), mask.copy()
    m1[..., 50:] = 0
    m2[..., :50] = 0
    o, lse = oracle.masked_attention(q, k, v, mask)
    o1, l1 = oracle.masked_attention(q, k, v, m1)
    o2, l2 = oracle.masked_attention(q, k, v, m2)
    m = np.maximum(l1, l2)
    w1, w2 = np.exp(l1 - m), np.exp(l2 - m)
    merged = (o1 * w1[..., None] + o2 * w2[..., None]) / (w1 + w2)[..., None]
    np.testing.assert_allclose(merged, o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(m + np.log(w1 + w2), lse, rtol=1e-12)


def test_appendix_a_error_bound_for_unrenormalised_output():
    """O - W Lambda V is bounded by (1 - kept mass) * max |v| (Appendix A); the kept mass of
    the dense softmax is exp(lse_kept - lse_all), and W Lambda V = kept mass * renormalised out."""
    q, k, v, mask = _rand(6)
    ones = np.ones_like(mask)
    o_all, lse_all = oracle.masked_attention(q, k, v, ones)
    o_sel, lse_sel = oracle.masked_attention(q, k, v, mask)
    kept = np.exp(lse_sel - lse_all)
    assert (kept <= 1 + 1e-12).all() and (kept > 0).all()
    err = np.abs(o_all - kept[..., None] * o_sel).max(axis=-1)
    vmax = np.abs(v).max()
    assert (err <= (1 - kept) * vmax + 1e-12).all()


def test_sequence_lengths_and_empty_rows():
    q, k, v, mask = _rand(7)
    lens = np.array([40, 97], dtype=np.int32)
    o, lse = oracle.masked_attention(q, k, v, mask, lens=lens)
    m2 = mask.copy()
    m2[0, :, 40:] = 0
    o2, lse2 = oracle.masked_attention(q, k, v, m2)
    np.testing.assert_array_equal(o, o2)
    np.testing.assert_array_equal(lse, lse2)
    empty = np.zeros_like(mask)
    o3, lse3 = oracle.masked_attention(q, k, v, empty)
    assert (o3 == 0).all() and np.isneginf(lse3).all()


def test_bf16_bit_inputs_equal_widened_inputs_and_row_subset():
    q, k, v, mask = _rand(8)
    qb, kb, vb = (W.round_to_bf16_bits(a).reshape(a.shape) for a in (q, k, v))
    qf, kf, vf = (W.bf16_bits_to_f32(a).reshape(a.shape) for a in (qb, kb, vb))
    o_bits, l_bits = oracle.masked_attention(qb, kb, vb, mask, bf16=True)
    o_f32, l_f32 = oracle.masked_attention(qf, kf, vf, mask)
    np.testing.assert_array_equal(o_bits, o_f32)
    np.testing.assert_array_equal(l_bits, l_f32)
    which = [(1, 5, 2), (0, 0, 0), (1, 7, 1)]
    o_w, l_w = oracle.masked_attention(qf, kf, vf, mask, which=which)
    for i, (b, h, t) in enumerate(which):
        np.testing.assert_array_equal(o_w[i], o_f32[b, h, t])
        assert l_w[i] == l_f32[b, h, t]
    # bf16 rounding helper: round-to-nearest-even agrees with torch's conversion
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(W.round_to_bf16_bits(x), want)


def test_custom_scale():
    q, k, v, mask = _rand(9)
    o, _ = oracle.masked_attention(q, k, v, mask, sm_scale=0.5)
    o_ref = _sdpa(q * np.float32(0.5 * np.sqrt(q.shape[-1])), k, v, mask)
    np.testing.assert_allclose(o, o_ref, rtol=1e-6, atol=1e-8)


# ---- the verifier's own new tokens behind the cache (causal tail) --------------------------------
def _tail(seed, B, H_kv, T, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, H_kv, T, d), dtype=np.float32),
            rng.standard_normal((B, H_kv, T, d), dtype=np.float32))


def _sdpa_tail(q, k, v, mask, k_new, v_new, lens=None):
    """Library route: one explicit boolean mask per query over [cache | new tokens]."""
    B, H_q, T, d = q.shape
    H_kv, n = k.shape[1], k.shape[2]
    G = H_q // H_kv
    tq = torch.from_numpy(q).double()
    tk = torch.from_numpy(np.concatenate([k, k_new], axis=2)).double().repeat_interleave(G, dim=1)
    tv = torch.from_numpy(np.concatenate([v, v_new], axis=2)).double().repeat_interleave(G, dim=1)
    am = np.zeros((B, H_kv, T, n + T), dtype=bool)
    for b in range(B):
        L = n if lens is None else int(lens[b])
        am[b, :, :, :L] = mask[b, :, None, :L].astype(bool)
        for t in range(T):
            am[b, :, t, n:n + t + 1] = True
    am = torch.from_numpy(am).repeat_interleave(G, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=am).numpy()


@pytest.mark.parametrize("shape", [dict(), dict(B=1, H_q=4, H_kv=4, T=5, d=64, n=130),
                                   dict(B=3, H_q=6, H_kv=3, T=1, d=8, n=33)])
def test_tail_equals_library_attention_with_per_query_mask(shape):
    q, k, v, mask = _rand(11, **shape)
    k_new, v_new = _tail(12, q.shape[0], k.shape[1], q.shape[2], q.shape[3])
    o, _ = oracle.masked_attention(q, k, v, mask, k_new=k_new, v_new=v_new)
    np.testing.assert_allclose(o, _sdpa_tail(q, k, v, mask, k_new, v_new), rtol=1e-10, atol=1e-12)


def test_tail_with_sequence_lengths_and_row_subset():
    q, k, v, mask = _rand(13, B=3, H_q=4, H_kv=2, T=4, d=16, n=50)
    lens = np.array([50, 0, 17], dtype=np.int32)
    k_new, v_new = _tail(14, 3, 2, 4, 16)
    o, _ = oracle.masked_attention(q, k, v, mask, lens=lens, k_new=k_new, v_new=v_new)
    np.testing.assert_allclose(o, _sdpa_tail(q, k, v, mask, k_new, v_new, lens), rtol=1e-10, atol=1e-12)
    which = [(2, 3, 1), (0, 0, 3), (1, 2, 0)]
    o_s, _ = oracle.masked_attention(q, k, v, mask, lens=lens, k_new=k_new, v_new=v_new, which=which)
    for i, (b, h, t) in enumerate(which):
        np.testing.assert_array_equal(o_s[i], o[b, h, t])


def test_tail_alone_first_query_returns_first_new_value_row():
    # empty cache: query 0 sees only new token 0, so its output is that token's value row and lse = its score
    q, k, v, _ = _rand(15, B=1, H_q=4, H_kv=2, T=3, d=16, n=9)
    k_new, v_new = _tail(16, 1, 2, 3, 16)
    none = np.zeros(k.shape[:3], dtype=np.uint8)
    o, lse = oracle.masked_attention(q, k, v, none, k_new=k_new, v_new=v_new)
    for h in range(4):
        np.testing.assert_allclose(o[0, h, 0], v_new[0, h // 2, 0], rtol=1e-12)
        s = float(q[0, h, 0].astype(np.float64) @ k_new[0, h // 2, 0].astype(np.float64)) / 4.0
        assert abs(lse[0, h, 0] - s) < 1e-12


def test_tail_is_causal_later_new_tokens_do_not_matter():
    q, k, v, mask = _rand(17, B=1, H_q=2, H_kv=1, T=4, d=8, n=20)
    k_new, v_new = _tail(18, 1, 1, 4, 8)
    o1, _ = oracle.masked_attention(q, k, v, mask, k_new=k_new, v_new=v_new)
    k2, v2 = k_new.copy(), v_new.copy()
    k2[:, :, 3], v2[:, :, 3] = 50.0, -9.0          # only query 3 may see new token 3
    o2, _ = oracle.masked_attention(q, k, v, mask, k_new=k2, v_new=v2)
    np.testing.assert_array_equal(o1[:, :, :3], o2[:, :, :3])
    assert np.abs(o1[:, :, 3] - o2[:, :, 3]).max() > 1e-3


def test_fp16_bit_inputs_equal_widened_inputs():
    q, k, v, mask = _rand(21, B=2, H_q=4, H_kv=2, T=3, d=16, n=60)
    k_new, v_new = _tail(22, 2, 2, 3, 16)
    h = [a.astype(np.float16) for a in (q, k, v, k_new, v_new)]
    h[1][0, 0, 5, 3] = np.float16(6.1e-5)          # smallest normal
    h[1][0, 0, 6, 3] = np.float16(6e-8)            # subnormal
    h[2][1, 1, 7, 0] = np.float16(-65504.0)        # largest magnitude
    wide = [a.astype(np.float32) for a in h]
    bits = [a.view(np.uint16) for a in h]
    o_w, l_w = oracle.masked_attention(wide[0], wide[1], wide[2], mask, k_new=wide[3], v_new=wide[4])
    o_b, l_b = oracle.masked_attention(bits[0], bits[1], bits[2], mask, f16=True, k_new=bits[3], v_new=bits[4])
    np.testing.assert_array_equal(o_w, o_b)
    np.testing.assert_array_equal(l_w, l_b)
