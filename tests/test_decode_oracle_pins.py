"""Pins for the decode-attention oracle: closed forms, invariants and library routines.

None compares the oracle with itself or with the HIP path; each names the mistake it catches.
"""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

from oracle import decode_oracle as dec


def rand(seed, B, Hq, Hkv, cap, D, scale=1.0):
    rng = np.random.default_rng(seed)
    q = (rng.standard_normal((B, Hq, D)) * scale).astype(np.float32)
    k = rng.standard_normal((B, Hkv, cap, D)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, cap, D)).astype(np.float32)
    return q, k, v


def test_zero_query_gives_the_mean_value_row():
    # catches: probabilities that do not sum to one, a wrong axis in the weighted sum
    q, k, v = rand(1, 2, 4, 2, 37, 16)
    q[:] = 0
    out, lse = dec.decode_attention(q, k, v)
    for b in range(2):
        for h in range(4):
            assert np.allclose(out[b, h], v[b, h // 2].astype(np.float64).mean(axis=0), rtol=0, atol=1e-14)
    assert np.allclose(lse, math.log(37.0), rtol=0, atol=1e-14)


def test_single_row_cache_returns_that_row():
    # catches: an off-by-one in the valid length, a normaliser that is not the row's own
    q, k, v = rand(2, 1, 2, 2, 5, 8)
    out, lse = dec.decode_attention(q, k, v, lens=1)
    assert np.array_equal(out[0], v[0, :, 0].astype(np.float64))
    want = np.einsum("hd,hd->h", q[0].astype(np.float64), k[0, :, 0].astype(np.float64)) / math.sqrt(8.0)
    assert np.allclose(lse[0], want, rtol=0, atol=1e-14)


def test_two_keys_against_the_logistic_function():
    # catches: a missing or wrong 1/sqrt(D) scale, a sign error in the exponent
    D = 4
    q = np.array([[[1.0, 2.0, -1.0, 0.5]]], dtype=np.float32)
    k = np.array([[[[0.5, 0.25, 1.0, 2.0], [-1.0, 1.5, 0.0, 1.0]]]], dtype=np.float32)
    v = np.array([[[[1.0, 0.0, 0.0, 0.0], [0.0, 1.0, 0.0, 0.0]]]], dtype=np.float32)
    s0 = (0.5 + 0.5 - 1.0 + 1.0) / 2.0      # q.k0 / sqrt(4), by hand
    s1 = (-1.0 + 3.0 + 0.0 + 0.5) / 2.0
    p0 = 1.0 / (1.0 + math.exp(s1 - s0))
    out, lse = dec.decode_attention(q, k, v)
    assert np.allclose(out[0, 0], [p0, 1.0 - p0, 0.0, 0.0], rtol=0, atol=1e-15)
    assert abs(lse[0, 0] - math.log(math.exp(s0) + math.exp(s1))) < 1e-15


def test_dominant_key_wins():
    # catches: softmax over the wrong axis, keys and values paired in different orders
    q, k, v = rand(3, 1, 2, 1, 64, 16)
    k[0, 0, 41] = q[0, 0] * 50.0
    out, _ = dec.decode_attention(q, k, v)
    assert np.allclose(out[0, 0], v[0, 0, 41], rtol=0, atol=1e-9)


def test_joint_row_permutation_changes_nothing():
    # the property that makes a compacted cache usable: only the set of kept rows matters.
    # catches: any dependence on position (a stray causal mask, positional weighting)
    q, k, v = rand(4, 2, 4, 4, 50, 8)
    perm = np.random.default_rng(0).permutation(50)
    a, la = dec.decode_attention(q, k, v)
    b, lb = dec.decode_attention(q, k[:, :, perm], v[:, :, perm])
    assert np.allclose(a, b, rtol=0, atol=1e-13) and np.allclose(la, lb, rtol=0, atol=1e-13)


def test_common_key_shift_changes_only_the_lse():
    # q.(k + c) = q.k + q.c for every row: the weights stay, the lse moves by q.c / sqrt(D).
    # catches: a maximum subtracted but not restored in the lse, an unstable exponential
    q, k, v = rand(5, 1, 2, 2, 33, 8)
    c = np.random.default_rng(1).standard_normal(8).astype(np.float32) * 30
    a, la = dec.decode_attention(q, k, v)
    b, lb = dec.decode_attention(q, (k.astype(np.float64) + c), v)
    assert np.allclose(a, b, rtol=0, atol=1e-10)
    assert np.allclose(lb - la, q[0].astype(np.float64) @ c.astype(np.float64) / math.sqrt(8.0), rtol=0, atol=1e-10)


def test_head_groups_read_their_own_kv_head():
    # catches: h % g instead of h // g, a transposed group layout
    B, Hq, Hkv, cap, D = 1, 6, 2, 9, 4
    q, k, v = rand(6, B, Hq, Hkv, cap, D)
    v[0, 0] = 1.0
    v[0, 1] = -2.0
    out, _ = dec.decode_attention(q, k, v)
    assert np.allclose(out[0, :3], 1.0, atol=1e-14) and np.allclose(out[0, 3:], -2.0, atol=1e-14)


def test_rows_beyond_the_valid_length_are_ignored():
    # catches: reading up to the capacity instead of the length, per-sequence lengths mixed up
    q, k, v = rand(7, 3, 2, 2, 40, 8)
    lens = [40, 7, 23]
    a, la = dec.decode_attention(q, k, v, lens=lens)
    k2, v2 = k.copy(), v.copy()
    for b, S in enumerate(lens):
        k2[b, :, S:] = 1e30
        v2[b, :, S:] = np.nan
    b_, lb = dec.decode_attention(q, k2, v2, lens=lens)
    assert np.array_equal(a, b_) and np.array_equal(la, lb)
    for b, S in enumerate(lens):
        c, _ = dec.decode_attention(q[b:b + 1], k[b:b + 1, :, :S], v[b:b + 1, :, :S])
        assert np.allclose(a[b], c[0], rtol=0, atol=1e-14)


def test_two_segments_merge_through_their_lse():
    # attention over A u B = the lse-weighted mix of attention over A and over B.
    # catches: an lse in the wrong base or missing the maximum; pins the second output
    q, k, v = rand(8, 2, 4, 2, 60, 8)
    full, lf = dec.decode_attention(q, k, v)
    a, la = dec.decode_attention(q, k[:, :, :25], v[:, :, :25])
    b, lb = dec.decode_attention(q, k[:, :, 25:], v[:, :, 25:])
    wa = 1.0 / (1.0 + np.exp(lb - la))
    assert np.allclose(full, wa[..., None] * a + (1 - wa[..., None]) * b, rtol=0, atol=1e-13)
    assert np.allclose(lf, np.logaddexp(la, lb), rtol=0, atol=1e-13)


def test_against_scipy_softmax_and_logsumexp():
    # a library routine for the same definition.  catches: anything the closed forms miss
    B, Hq, Hkv, cap, D = 2, 8, 4, 77, 16
    q, k, v = rand(9, B, Hq, Hkv, cap, D, scale=3.0)
    out, lse = dec.decode_attention(q, k, v)
    g = Hq // Hkv
    kk = np.repeat(k.astype(np.float64), g, axis=1)
    vv = np.repeat(v.astype(np.float64), g, axis=1)
    s = np.einsum("bhd,bhjd->bhj", q.astype(np.float64), kk) / math.sqrt(D)
    assert np.allclose(out, np.einsum("bhj,bhjd->bhd", softmax(s, axis=-1), vv), rtol=0, atol=1e-13)
    assert np.allclose(lse, logsumexp(s, axis=-1), rtol=0, atol=1e-13)


def test_bf16_and_half_storage_are_widened_exactly():
    # catches: a lossy conversion of the stored values before the arithmetic
    q, k, v = rand(10, 1, 2, 2, 12, 8)
    tb = lambda a: torch.from_numpy(a).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    a, _ = dec.decode_attention(bits(tb(q)), bits(tb(k)), bits(tb(v)))
    b, _ = dec.decode_attention(tb(q).double().numpy(), tb(k).double().numpy(), tb(v).double().numpy())
    assert np.array_equal(a, b)
    c, _ = dec.decode_attention(q.astype(np.float16), k.astype(np.float16), v.astype(np.float16))
    d, _ = dec.decode_attention(q.astype(np.float16).astype(np.float64), k.astype(np.float16).astype(np.float64),
                                v.astype(np.float16).astype(np.float64))
    assert np.array_equal(c, d)


def test_bad_lengths_are_refused():
    q, k, v = rand(11, 1, 2, 2, 5, 4)
    with pytest.raises(ValueError):
        dec.decode_attention(q, k, v, lens=0)
    with pytest.raises(ValueError):
        dec.decode_attention(q, k, v, lens=6)
