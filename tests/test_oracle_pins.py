"""Pins for the fp64 oracle: closed forms, invariants, library special cases, brute force.

None of these compares the oracle with itself or with the HIP path.  Each pin names the
mistake it is meant to catch.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import snapkv_oracle as orc
from oracle import c_oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, Hq, Hkv, L, D, W, dtype="f32"):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((Hq, W, D)).astype(np.float32)
    k = rng.standard_normal((Hkv, L, D)).astype(np.float32)
    v = rng.standard_normal((Hkv, L, D)).astype(np.float32)
    if dtype == "bf16":
        f = lambda a: (torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy()
                       .view(np.uint16))
        return f(q), f(k), f(v)
    return q, k, v


# ----------------------------------------------------------------------------- storage
def test_widen_bf16_is_exact():
    # catches: a wrong shift or byte order when decoding bf16
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x3DCD, 0x7F80], dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.widen(bits), want)
    assert orc.widen(bits)[0] == 1.0 and orc.widen(bits)[1] == -2.0


# ----------------------------------------------------------------------------- softmax / mask
@pytest.mark.parametrize("L,W,D", [(40, 8, 16), (33, 32, 8), (17, 1, 4)])
def test_rows_sum_to_one_and_mask_shape(L, W, D):
    # catches: missing normalisation, mask off by one, mask applied to prefix columns
    q, k, _ = rand_case(1, 1, 1, L, D, W)
    P = orc.window_probs(q[0], k[0])
    n = L - W
    assert P.shape == (W, L)
    assert np.allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    for i in range(W):
        assert np.all(P[i, :n + i + 1] > 0.0)
        assert np.all(P[i, n + i + 1:] == 0.0)


def test_mass_conservation():
    # vote mass on the prefix plus the mass the rows put on window columns equals W
    q, k, _ = rand_case(2, 1, 1, 64, 16, 8)
    P = orc.window_probs(q[0], k[0])
    vt = orc.vote(P)
    assert vt.shape == (56,)
    assert abs(vt.sum() + P[:, 56:].sum() - 8.0) < 1e-12


def test_two_key_closed_form():
    # one query, two visible keys: probabilities are the logistic function of the logit gap.
    # catches: dropped 1/sqrt(D) scale, transposed operands, wrong exponent sign
    D = 4
    q = np.array([[[1.0, 2.0, -1.0, 0.5]]], dtype=np.float32)        # W=1
    k = np.array([[[0.5, 0.25, 1.0, 2.0], [1.0, -1.0, 0.0, 3.0]]], dtype=np.float32)  # L=2
    s0 = (0.5 + 0.5 - 1.0 + 1.0) / math.sqrt(D)
    s1 = (1.0 - 2.0 + 0.0 + 1.5) / math.sqrt(D)
    P = orc.window_probs(q[0], k[0])
    assert P.shape == (1, 2)
    assert abs(P[0, 0] - 1.0 / (1.0 + math.exp(s1 - s0))) < 1e-15
    assert abs(orc.vote(P)[0] - P[0, 0]) == 0.0


def test_widen_fp16_is_exact():
    # IEEE half values, including a subnormal and the largest finite one, written out by hand
    x = np.array([1.0, -2.5, 2.0 ** -24, 65504.0, 0.333251953125], dtype=np.float16)
    assert orc.widen(x).tolist() == [1.0, -2.5, 2.0 ** -24, 65504.0, 0.333251953125]
    q, k, v = rand_case(9, 2, 2, 40, 8, 4)
    a = orc.compress(q.astype(np.float16), k.astype(np.float16), v.astype(np.float16), 4, 0, 3, 12)
    b = orc.compress(q.astype(np.float16).astype(np.float32), k.astype(np.float16).astype(np.float32),
                     v.astype(np.float16).astype(np.float32), 4, 0, 3, 12)
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[4], b[4]) and a[0].dtype == np.float16


# ----------------------------------------------------------------------------- closed form: zero queries
def harmonic_gap(L, n):
    return float(sum(Fraction(1, t) for t in range(n + 1, L + 1)))


@pytest.mark.parametrize("L,W", [(64, 8), (100, 32), (50, 1)])
def test_zero_queries_votes_are_harmonic(L, W):
    # row i is uniform over n+i+1 keys, so every prefix vote is H_L - H_n.
    # catches: causal mask off by one, summing W+1 or W-1 rows (Eq. 1's printed limit)
    D = 8
    q = np.zeros((1, W, D), dtype=np.float32)
    _, k, _ = rand_case(3, 1, 1, L, D, W)
    vt = orc.vote(orc.window_probs(q[0], k[0]))
    assert np.allclose(vt, harmonic_gap(L, L - W), rtol=1e-13, atol=0)


def test_zero_queries_maxpool_selects_lowest_indices():
    # all pooled scores equal -> the tie rule alone decides: positions 0..k-1
    L, W, D, C, p = 96, 16, 8, 40, 7
    q = np.zeros((2, W, D), dtype=np.float32)
    _, k, v = rand_case(4, 2, 2, L, D, W)
    _, _, idx, kept, score = orc.compress(q, k, v, W, orc.POOL_MAX, p, C)
    assert kept == C
    assert np.all(score == score[0, 0])          # flat field, bit-identical
    want = np.concatenate([np.arange(C - W), np.arange(L - W, L)])
    assert np.array_equal(idx[0], want) and np.array_equal(idx[1], want)


def test_zero_queries_avgpool_edges_count_padding():
    # average pooling divides by p even at the edges, so the p//2 edge positions score lower:
    # the selection starts at p//2.  catches: dividing by the number of in-range taps
    L, W, D, C, p = 96, 16, 8, 40, 5
    q = np.zeros((1, W, D), dtype=np.float32)
    _, k, v = rand_case(5, 1, 1, L, D, W)
    _, _, idx, _, score = orc.compress(q, k, v, W, orc.POOL_AVG, p, C)
    h = harmonic_gap(L, L - W)
    n = L - W
    assert np.allclose(score[0, 2:n - 2], h, rtol=1e-13)
    assert np.allclose(score[0, [0, n - 1]], h * 3 / 5, rtol=1e-13)
    assert np.allclose(score[0, [1, n - 2]], h * 4 / 5, rtol=1e-13)
    # interior values are sums of five equal numbers / 5; tiny rounding differences may exist,
    # so only check that no edge position was selected and that the set is a contiguous run
    sel = idx[0, :C - W]
    assert sel.min() >= 2 and sel.max() <= n - 3
    assert len(set(sel.tolist())) == C - W


# ----------------------------------------------------------------------------- pooling
def _golden_pool():
    rows = {}
    with open(os.path.join(GOLDEN, "pool_small.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *vals = line.split()
            rows[name] = np.array([float(x) for x in vals])
    return rows


def test_pool_hand_worked():
    # catches: wrong reach (p vs p//2), wrong edge handling, wrong avg divisor
    g = _golden_pool()
    x = g["x"]
    for fn in (orc.pool1d, orc._pool1d_fast):
        assert np.array_equal(fn(x, orc.POOL_MAX, 3), g["max3"])
        assert np.array_equal(fn(x, orc.POOL_MAX, 5), g["max5"])
        assert np.allclose(fn(x, orc.POOL_AVG, 3), g["avg3x3"] / 3, rtol=1e-15)
        assert np.allclose(fn(x, orc.POOL_AVG, 5), g["avg5x5"] / 5, rtol=1e-15)
        assert np.array_equal(fn(x, orc.POOL_MAX, 1), x)
        assert np.array_equal(fn(x, orc.POOL_AVG, 1), x)


@pytest.mark.parametrize("p", [1, 3, 5, 7, 13])
@pytest.mark.parametrize("kind", [0, 1])
def test_pool_matches_library_routine(p, kind):
    # torch's pooling with padding=p//2, stride 1 is the routine Listing 1 names
    rng = np.random.default_rng(6)
    x = rng.random(57)
    t = torch.from_numpy(x)[None, None, :]
    if kind == 0:
        want = torch.nn.functional.max_pool1d(t, p, stride=1, padding=p // 2)[0, 0].numpy()
        assert np.array_equal(orc.pool1d(x, kind, p), want)
        assert np.array_equal(orc._pool1d_fast(x, kind, p), want)
    else:
        want = torch.nn.functional.avg_pool1d(t, p, stride=1, padding=p // 2,
                                              count_include_pad=True)[0, 0].numpy()
        assert np.allclose(orc.pool1d(x, kind, p), want, rtol=1e-14)
        assert np.allclose(orc._pool1d_fast(x, kind, p), want, rtol=1e-14)


def test_even_kernel_rejected():
    with pytest.raises(ValueError):
        orc.pool1d(np.ones(8), 0, 4)


# ----------------------------------------------------------------------------- selection
def test_select_tie_rule_hand_worked():
    # catches: ties going to the higher index, output in score order instead of position order
    s = np.array([1.0, 3.0, 3.0, 2.0, 3.0, 0.5])
    assert orc.select(s, 2).tolist() == [1, 2]
    assert orc.select(s, 3).tolist() == [1, 2, 4]
    assert orc.select(s, 4).tolist() == [1, 2, 3, 4]
    assert orc.select(s, 0).tolist() == []
    assert orc.select(s, 6).tolist() == [0, 1, 2, 3, 4, 5]


def test_w1_p1_equals_plain_sort_of_logits():
    # one attention row, no pooling: softmax is monotone, so the kept set is the top-(C-1)
    # raw dot products.  catches: selecting smallest, selecting over window columns
    L, D, C = 48, 8, 12
    q, k, v = rand_case(7, 1, 1, L, D, 1)
    _, _, idx, _, _ = orc.compress(q, k, v, 1, orc.POOL_MAX, 1, C)
    logits = [sum(float(q[0, 0, d]) * float(k[0, j, d]) for d in range(D)) for j in range(L - 1)]
    best = sorted(range(L - 1), key=lambda j: (-logits[j], j))[:C - 1]
    assert idx[0].tolist() == sorted(best) + [L - 1]


def test_nested_and_value_independent():
    q, k, v = rand_case(8, 2, 2, 80, 16, 8)
    _, _, big, _, _ = orc.compress(q, k, v, 8, orc.POOL_MAX, 3, 40)
    _, _, small, _, _ = orc.compress(q, k, v, 8, orc.POOL_MAX, 3, 24)
    _, _, other_v, _, _ = orc.compress(q, k, -3.0 * v + 1.0, 8, orc.POOL_MAX, 3, 40)
    for h in range(2):
        assert set(small[h].tolist()) <= set(big[h].tolist())
    assert np.array_equal(big, other_v)


# ----------------------------------------------------------------------------- invariants of the output
@pytest.mark.parametrize("kind,p", [(0, 7), (1, 5), (0, 1)])
def test_output_invariants(kind, p):
    L, W, D, C = 120, 16, 16, 48
    q, k, v = rand_case(9, 4, 2, L, D, W)
    ok, ov, idx, kept, score = orc.compress(q, k, v, W, kind, p, C)
    assert kept == C and idx.shape == (2, C) and ok.shape == (2, C, D)
    for h in range(2):
        assert np.all(np.diff(idx[h]) > 0)                       # unique and ascending
        assert idx[h, 0] >= 0 and idx[h, -1] == L - 1
        assert np.array_equal(idx[h, C - W:], np.arange(L - W, L))   # window kept
        assert np.array_equal(ok[h], k[h][idx[h]]) and np.array_equal(ov[h], v[h][idx[h]])
    assert np.all(score >= 0.0)


@pytest.mark.parametrize("L,C", [(32, 32), (20, 64), (33, 40)])
def test_bypass_identity(L, C):
    q, k, v = rand_case(10, 2, 2, L, 8, 8)
    ok, ov, idx, kept, score = orc.compress(q, k, v, 8, 0, 3, C)
    assert kept == L and score is None
    assert np.array_equal(ok, k) and np.array_equal(ov, v)
    assert np.array_equal(idx, np.tile(np.arange(L), (2, 1)))


def test_l_equals_c_plus_one_drops_exactly_one():
    L, W, D = 41, 8, 8
    q, k, v = rand_case(11, 1, 1, L, D, W)
    _, _, idx, kept, score = orc.compress(q, k, v, W, 0, 1, 40)
    dropped = set(range(L)) - set(idx[0].tolist())
    assert kept == 40 and len(dropped) == 1
    assert dropped == {int(np.argmin(score[0]))}      # random scores: no ties


# ----------------------------------------------------------------------------- invariances
def test_shift_invariance_large_offset():
    # adding one vector to every key shifts whole rows of logits; a huge offset also checks
    # the max subtraction (a naive exp would overflow)
    L, W, D = 96, 8, 16
    q, k, v = rand_case(12, 1, 1, L, D, W)
    c = np.full((D,), 300.0, dtype=np.float32) * np.sign(q[0].sum(axis=0))
    s0 = orc.pooled_scores(q, k.astype(np.float64), W, 0, 1)
    s1 = orc.pooled_scores(q, k.astype(np.float64) + c.astype(np.float64), W, 0, 1)
    assert np.all(np.isfinite(s1))
    assert np.allclose(s0, s1, rtol=1e-9, atol=0)


def test_permutation_equivariance_p1():
    L, W, D, C = 72, 8, 16, 24
    q, k, v = rand_case(13, 1, 1, L, D, W)
    rng = np.random.default_rng(0)
    perm = rng.permutation(L - W)
    k2, v2 = k.copy(), v.copy()
    k2[0, :L - W] = k[0, perm]
    v2[0, :L - W] = v[0, perm]
    _, _, i1, _, s1 = orc.compress(q, k, v, W, 0, 1, C)
    _, _, i2, _, s2 = orc.compress(q, k2, v2, W, 0, 1, C)
    assert np.allclose(s2[0], s1[0][perm], rtol=1e-12)
    assert set(perm[i2[0, :C - W]].tolist()) == set(i1[0, :C - W].tolist())


def test_planted_one_hot_key_and_pool_reach():
    # a key aligned with the mean window query and scaled up takes nearly all the mass of
    # every row: its vote is ~W, max pooling spreads that to +-p//2 and all of them are kept
    L, W, D, C, p = 200, 8, 16, 24, 7
    rng = np.random.default_rng(14)
    base = rng.standard_normal(D)
    q = (base[None, None, :] + 0.05 * rng.standard_normal((1, W, D))).astype(np.float32)
    k = (0.1 * rng.standard_normal((1, L, D))).astype(np.float32)
    v = rng.standard_normal((1, L, D)).astype(np.float32)
    pos = 77
    k[0, pos] = (40.0 * base / np.linalg.norm(base)).astype(np.float32)
    _, _, idx, _, score = orc.compress(q, k, v, W, orc.POOL_MAX, p, C)
    assert abs(score[0, pos] - W) < 1e-6
    assert np.all(score[0, pos - 3:pos + 4] == score[0, pos])
    assert score[0, pos - 4] < 1e-3 and score[0, pos + 4] < 1e-3
    assert set(range(pos - 3, pos + 4)) <= set(idx[0].tolist())


# ----------------------------------------------------------------------------- library routines (MHA)
@pytest.mark.parametrize("kind,p", [(0, 7), (1, 5)])
def test_mha_matches_torch_cpu_routines(kind, p):
    # for MHA the listing is matmul / softmax / sum / pool1d / topk / gather / cat; run those
    # library calls in fp64 on a small input as a second, independently written opinion
    H, L, W, D, C = 3, 90, 16, 32, 40
    q, k, v = rand_case(15, H, H, L, D, W)
    tq, tk, tv = (torch.from_numpy(a).double() for a in (q, k, v))
    n = L - W
    att = tq @ tk.transpose(1, 2) / math.sqrt(D)
    mask = torch.full((W, W), float("-inf")).triu(1)
    att[:, :, n:] += mask
    att = torch.softmax(att, dim=-1)
    vt = att[:, :, :n].sum(dim=1)
    if kind == 0:
        pv = torch.nn.functional.max_pool1d(vt[None], p, stride=1, padding=p // 2)[0]
    else:
        pv = torch.nn.functional.avg_pool1d(vt[None], p, stride=1, padding=p // 2)[0]
    top = pv.topk(C - W, dim=-1).indices
    gk = torch.cat([tk[:, :n].gather(1, top[..., None].expand(-1, -1, D)), tk[:, n:]], dim=1)

    ok, ov, idx, kept, score = orc.compress(q, k, v, W, kind, p, C)
    assert np.allclose(score, pv.numpy(), rtol=1e-12, atol=0)
    for h in range(H):
        # sets only: topk's order and tie choice are the library's own
        s_lib = pv[h].numpy()
        thr = np.sort(s_lib)[::-1][C - W - 1]
        strict = set(np.nonzero(s_lib > thr)[0].tolist())
        assert strict <= set(idx[h, :C - W].tolist())
        assert np.all(s_lib[idx[h, :C - W]] >= thr)
        if len(strict) == C - W - 1 or (s_lib == thr).sum() == 1:
            assert set(top[h].tolist()) == set(idx[h, :C - W].tolist())
    # gathered rows: where the library's tie choice gave the same set, its gather+cat holds the
    # same rows; ordered by position they equal the oracle's output exactly
    checked = 0
    for h in range(H):
        lib_set, orc_set = set(top[h].tolist()), set(idx[h, :C - W].tolist())
        if lib_set != orc_set:
            # the two may differ only in which of the positions tied at the threshold they took
            s_lib = pv[h].numpy()
            thr = np.sort(s_lib)[::-1][C - W - 1]
            assert all(s_lib[j] == thr for j in lib_set ^ orc_set)
            continue
        order = torch.argsort(top[h])
        lib_rows = torch.cat([gk[h, :C - W][order], gk[h, C - W:]], dim=0).numpy()
        assert np.array_equal(orc.widen(ok[h]), lib_rows)
        checked += 1
    assert checked >= 1 or kind == 0      # max pooling routinely ties at the threshold


# ----------------------------------------------------------------------------- GQA convention
def test_gqa_is_pool_then_sum_over_group():
    # a KV head's score is the sum of the scores its query heads would get on their own
    # (each pooled separately); differs from pooling the summed votes under max pooling
    L, W, D, p = 70, 8, 16, 5
    q, k, v = rand_case(16, 4, 2, L, D, W)
    got = orc.pooled_scores(q, k, W, orc.POOL_MAX, p)
    for hk in range(2):
        parts = [orc.pooled_scores(q[h:h + 1], k[hk:hk + 1], W, orc.POOL_MAX, p)[0]
                 for h in (2 * hk, 2 * hk + 1)]
        assert np.allclose(got[hk], parts[0] + parts[1], rtol=1e-15)
        votes = [orc.vote(orc.window_probs(q[h], k[hk])) for h in (2 * hk, 2 * hk + 1)]
        other = orc.pool1d(votes[0] + votes[1], orc.POOL_MAX, p)
        assert not np.allclose(got[hk], other, rtol=1e-6)


# ----------------------------------------------------------------------------- brute force, pure Python loops
def brute_force(q, k, v, Hq, Hkv, L, D, W, kind, p, C):
    g = Hq // Hkv
    n = L - W
    out = []
    for hk in range(Hkv):
        score = [0.0] * n
        for h in range(hk * g, (hk + 1) * g):
            vt = [0.0] * n
            for i in range(W):
                vis = n + i + 1
                s = [sum(float(q[h][i][d]) * float(k[hk][j][d]) for d in range(D)) / math.sqrt(D)
                     for j in range(vis)]
                m = max(s)
                e = [math.exp(x - m) for x in s]
                z = math.fsum(e)
                for j in range(n):
                    vt[j] += e[j] / z
            r = p // 2
            for j in range(n):
                taps = [vt[t] for t in range(j - r, j + r + 1) if 0 <= t < n]
                score[j] += max(taps) if kind == 0 else sum(taps) / p
        order = sorted(range(n), key=lambda j: (-score[j], j))[:C - W]
        out.append((score, sorted(order) + list(range(n, L))))
    return out


@pytest.mark.parametrize("Hq,Hkv,L,D,W,kind,p,C,dtype", [
    (2, 2, 40, 8, 4, 0, 3, 16, "f32"),
    (4, 2, 64, 8, 8, 1, 5, 24, "f32"),
    (4, 1, 48, 16, 6, 0, 7, 20, "bf16"),
    (1, 1, 30, 4, 1, 0, 1, 10, "bf16"),
])
def test_brute_force_three_writings(Hq, Hkv, L, D, W, kind, p, C, dtype):
    q, k, v = rand_case(17 + L, Hq, Hkv, L, D, W, dtype)
    qf, kf = orc.widen(q), orc.widen(k)
    want = brute_force(qf, kf, None, Hq, Hkv, L, D, W, kind, p, C)
    ok, ov, idx, kept, score = orc.compress(q, k, v, W, kind, p, C)
    ck, cv, cidx, ckept, cscore = c_oracle.compress(q, k, v, W, kind, p, C)
    assert kept == ckept == C
    for hk in range(Hkv):
        assert np.allclose(score[hk], want[hk][0], rtol=1e-12, atol=0)
        assert np.allclose(cscore[hk], want[hk][0], rtol=1e-12, atol=0)
        assert idx[hk].tolist() == want[hk][1]
        assert cidx[hk].tolist() == want[hk][1]
    assert np.array_equal(ok, ck) and np.array_equal(ov, cv)
    assert ok.dtype == k.dtype


# ----------------------------------------------------------------------------- handed-in log-sum-exp
def test_lse_two_key_closed_form():
    # one query, two visible keys: lse = log(e^s0 + e^s1), written out by hand.
    # catches: a missing scale, a base-2 / base-e mix-up, max-subtraction left in the result
    D = 4
    q = np.array([[1.0, 2.0, -1.0, 0.5]], dtype=np.float32)
    k = np.array([[0.5, 0.25, 1.0, 2.0], [1.0, -1.0, 0.0, 3.0]], dtype=np.float32)
    s0 = (0.5 + 0.5 - 1.0 + 1.0) / math.sqrt(D)
    s1 = (1.0 - 2.0 + 0.0 + 1.5) / math.sqrt(D)
    lse = orc.window_lse(q, k)
    assert lse.shape == (1,)
    assert abs(lse[0] - math.log(math.exp(s0) + math.exp(s1))) < 1e-15
    P = orc.window_probs_given_lse(q, k, lse)
    assert abs(P[0, 0] - math.exp(s0) / (math.exp(s0) + math.exp(s1))) < 1e-15


def test_lse_matches_library_logsumexp_over_visible_keys():
    # catches: the causal mask missing from (or off by one in) the log-sum-exp
    from scipy.special import logsumexp
    W, L, D = 6, 40, 8
    q, k, _ = rand_case(61, 1, 1, L, D, W)
    lse = orc.window_lse(q[0], k[0])
    s = (q[0].astype(np.float64) @ k[0].astype(np.float64).T) / math.sqrt(D)
    for i in range(W):
        assert abs(lse[i] - logsumexp(s[i, : L - W + i + 1])) < 1e-13


@pytest.mark.parametrize("dtype,kind,p", [("f32", 0, 7), ("bf16", 1, 5)])
def test_true_lse_reproduces_the_softmax_path(dtype, kind, p):
    # handing in the rows' own log-sum-exp must change nothing: same scores, same kept positions
    Hq, Hkv, L, D, W, C = 4, 2, 300, 16, 16, 60
    q, k, v = rand_case(62, Hq, Hkv, L, D, W, dtype)
    lse = np.stack([orc.window_lse(q[h], k[h // 2]) for h in range(Hq)])
    for h in range(Hq):
        assert np.allclose(orc.window_probs_given_lse(q[h], k[h // 2], lse[h]), orc.window_probs(q[h], k[h // 2]),
                           rtol=1e-12, atol=1e-300)
    a = orc.compress(q, k, v, W, kind, p, C)
    b = orc.compress(q, k, v, W, kind, p, C, lse=lse)
    assert np.allclose(a[4], b[4], rtol=1e-12, atol=0)
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_lse_offset_scales_each_row():
    # raising row i's lse by d_i scales that row's probabilities by exp(-d_i): the votes become the
    # correspondingly weighted column sum.  catches: lse applied per column, or with the wrong sign
    W, L, D = 5, 64, 8
    q, k, _ = rand_case(63, 1, 1, L, D, W)
    lse = orc.window_lse(q[0], k[0])
    d = np.array([0.0, math.log(2.0), -0.5, 3.0, 1.25])
    P = orc.window_probs(q[0], k[0])
    got = orc.vote(orc.window_probs_given_lse(q[0], k[0], lse + d))
    want = (P[:, : L - W] * np.exp(-d)[:, None]).sum(axis=0)
    assert np.allclose(got, want, rtol=1e-13, atol=0)
    # a common offset rescales every vote alike and cannot change the selection
    s0 = orc.pooled_scores(q, k, W, 0, 3)
    s1 = orc.pooled_scores(q, k, W, 0, 3, lse=(lse + math.log(2.0))[None, :])
    assert np.allclose(s1, 0.5 * s0, rtol=1e-13, atol=0)
    assert np.array_equal(orc.select(s0[0], 10), orc.select(s1[0], 10))


# ----------------------------------------------------------------------------- C oracle vs numpy oracle, larger
@pytest.mark.parametrize("dtype,kind,p,W", [("bf16", 0, 7, 32), ("f32", 1, 5, 16), ("bf16", 0, 13, 64)])
def test_c_and_numpy_oracles_agree(dtype, kind, p, W):
    Hq, Hkv, L, D, C = 8, 4, 700, 64, 160
    q, k, v = rand_case(40 + W, Hq, Hkv, L, D, W, dtype)
    ok, ov, idx, kept, score = orc.compress(q, k, v, W, kind, p, C)
    ck, cv, cidx, ckept, cscore = c_oracle.compress(q, k, v, W, kind, p, C)
    assert np.allclose(score, cscore, rtol=1e-12, atol=0)
    assert np.array_equal(idx, cidx)
    assert np.array_equal(ok, ck) and np.array_equal(ov, cv)
    assert np.allclose(c_oracle.pooled_scores(q, k, W, kind, p), score, rtol=1e-12)


def test_c_oracle_bypass_and_errors():
    q, k, v = rand_case(50, 2, 2, 24, 8, 8)
    ck, cv, cidx, kept, score = c_oracle.compress(q, k, v, 8, 0, 3, 32)
    assert kept == 24 and score is None
    assert np.array_equal(ck, k) and np.array_equal(cidx, np.tile(np.arange(24), (2, 1)))
    with pytest.raises(ValueError):
        c_oracle.pooled_scores(q, k, 8, 0, 4)
    assert c_oracle.threads() >= 1


# ----------------------------------------------------------------------------- one cache per query head
def test_per_query_head_form_solves_each_head_alone():
    # catches: h % g instead of h // g in the head mapping, any leakage between query heads
    Hq, Hkv, L, D, W, C = 6, 2, 90, 8, 4, 20
    q, k, v = rand_case(41, Hq, Hkv, L, D, W)
    ok, ov, oi, kept, sc = orc.compress_per_query_head(q, k, v, W, orc.POOL_MAX, 3, C)
    assert ok.shape == (Hq, C, D) and oi.shape == (Hq, C) and kept == C
    for h in range(Hq):
        hk = h // (Hq // Hkv)
        a = orc.compress(q[h:h + 1], k[hk:hk + 1], v[hk:hk + 1], W, orc.POOL_MAX, 3, C)
        assert np.array_equal(oi[h], a[2][0]) and np.array_equal(ok[h], a[0][0]) and np.array_equal(ov[h], a[1][0])
        assert np.array_equal(sc[h], a[4][0])


def test_per_query_head_form_equals_the_grouped_form_without_groups():
    q, k, v = rand_case(42, 4, 4, 70, 8, 4)
    a = orc.compress_per_query_head(q, k, v, 4, orc.POOL_AVG, 5, 16)
    b = orc.compress(q, k, v, 4, orc.POOL_AVG, 5, 16)
    assert all(np.array_equal(x, y) for x, y in zip(a[:3], b[:3])) and a[3] == b[3]


def test_per_query_head_form_keeps_what_each_head_looks_for():
    # two query heads of one group look for different planted keys: each keeps its own, the
    # grouped form keeps both.  catches: a sum over the group left in the per-head form
    Hq, Hkv, L, D, W, C = 2, 1, 64, 8, 2, 3
    q = np.zeros((Hq, W, D), dtype=np.float32)
    k = np.zeros((Hkv, L, D), dtype=np.float32)
    v = np.arange(Hkv * L * D, dtype=np.float32).reshape(Hkv, L, D)
    q[0, :, 0] = 30.0
    q[1, :, 1] = 30.0
    k[0, 10, 0] = 1.0
    k[0, 40, 1] = 1.0
    _, _, oi, _, _ = orc.compress_per_query_head(q, k, v, W, orc.POOL_MAX, 1, C)
    assert oi[0].tolist() == [10, 62, 63] and oi[1].tolist() == [40, 62, 63]
    _, _, og, _, _ = orc.compress(q, k, v, W, orc.POOL_MAX, 1, 4)
    assert og[0].tolist() == [10, 40, 62, 63]


# ----------------------------------------------------------------------------- rate-form capacity
def test_capacity_for_rate_closed_cases():
    # catches: rounding up or to nearest instead of down, the rate applied to L instead of L - W
    assert orc.capacity_for_rate(1000, 32, 0.0) == 32
    assert orc.capacity_for_rate(1000, 32, 1.0) == 1000
    assert orc.capacity_for_rate(1032, 32, 0.5) == 32 + 500
    assert orc.capacity_for_rate(1033, 32, 0.5) == 32 + 500          # floor(500.5)
    assert orc.capacity_for_rate(132, 32, 0.25) == 32 + 25
    assert orc.capacity_for_rate(35, 32, 0.999) == 32 + 2            # floor(2.997)
    for n in (1, 7, 100, 4096):
        for num, den in ((1, 2), (1, 4), (3, 8), (5, 16)):           # dyadic rates: the product is exact
            assert orc.capacity_for_rate(n + 16, 16, num / den) == 16 + (n * num) // den
    with pytest.raises(ValueError):
        orc.capacity_for_rate(100, 32, 1.5)


# ----------------------------------------------------------------------------- hit rate (Eq. 3-7)
def test_hit_rate_uniform_attention():
    # zero query: A_cur = 1/Lk everywhere.  Below that value every prefix position is important and
    # the hits are the selected ones; above it nothing is.  catches: >= instead of >, a wrong denominator
    Hq, Hkv, Lk, n, D = 4, 2, 50, 40, 8
    q = np.zeros((Hq, D), dtype=np.float32)
    k = np.random.default_rng(3).standard_normal((Hkv, Lk, D)).astype(np.float32)
    A = orc.current_attention(q, k)
    assert np.allclose(A, 1.0 / Lk, rtol=0, atol=1e-16) and A.shape == (Hq, Lk)
    idx = np.array([[1, 5, 9], [0, 2, 39]])
    imp, hits = orc.hit_rate_counts(A[:, :n], idx, 0.5 / Lk)
    assert imp.tolist() == [n] * Hq and hits.tolist() == [3] * Hq
    assert orc.hit_rate(imp, hits) == 3 / n
    imp, hits = orc.hit_rate_counts(A[:, :n], idx, 1.0 / Lk + 1e-12)
    assert imp.sum() == 0 and hits.sum() == 0 and np.isnan(orc.hit_rate(imp, hits))
    imp, hits = orc.hit_rate_counts(np.full((Hq, n), 0.25), idx, 0.25)      # equality is not above
    assert imp.sum() == 0


def test_hit_rate_planted_keys_hand_counted():
    # head 0 looks at keys 3 and 20, head 1 at key 7 and at key 45, which lies outside the prefix
    Hq, Hkv, Lk, n, D = 2, 2, 48, 40, 4
    q = np.zeros((Hq, D), dtype=np.float32)
    k = np.zeros((Hkv, Lk, D), dtype=np.float32)
    q[0, 0] = 20.0
    q[1, 1] = 20.0
    k[0, 3, 0] = k[0, 20, 0] = 1.0
    k[1, 7, 1] = k[1, 45, 1] = 1.0
    A = orc.current_attention(q, k)
    assert abs(A[0, 3] - 0.5) < 1e-3 and abs(A[1, 45] - 0.5) < 1e-3 and np.allclose(A.sum(axis=1), 1.0)
    idx = np.array([[3, 4], [8, 9]])                 # head 0 kept one of its two keys, head 1 none
    imp, hits = orc.hit_rate_counts(A[:, :n], idx, 0.1)
    assert imp.tolist() == [2, 1] and hits.tolist() == [1, 0]
    assert orc.hit_rate(imp, hits) == 1 / 3


def test_hit_rate_counts_against_python_sets():
    # catches: a group mapping that is not h // g, masks built on the wrong axis
    rng = np.random.default_rng(8)
    Hq, Hkv, n = 6, 3, 30
    A = rng.random((Hq, n)) * 0.1
    idx = np.stack([np.sort(rng.choice(n, size=7, replace=False)) for _ in range(Hkv)])
    imp, hits = orc.hit_rate_counts(A, idx, 0.05)
    for h in range(Hq):
        important = {j for j in range(n) if A[h, j] > 0.05}
        assert imp[h] == len(important) and hits[h] == len(important & set(idx[h // 2].tolist()))
    idx_q = np.stack([np.sort(rng.choice(n, size=5, replace=False)) for _ in range(Hq)])
    imp2, hits2 = orc.hit_rate_counts(A, idx_q, 0.05)
    for h in range(Hq):
        assert hits2[h] == len({j for j in range(n) if A[h, j] > 0.05} & set(idx_q[h].tolist()))
    assert np.array_equal(imp, imp2)


def test_current_attention_is_the_decoding_softmax():
    # the same weights the decoding oracle (pinned on its own) applies to the value rows
    from oracle import decode_oracle as dec
    rng = np.random.default_rng(9)
    Hq, Hkv, Lk, D = 4, 2, 16, 16            # Lk = D so that one-hot rows fit the value tensor
    q = rng.standard_normal((Hq, D)).astype(np.float32)
    k = rng.standard_normal((Hkv, Lk, D)).astype(np.float32)
    A = orc.current_attention(q, k)
    eye = np.broadcast_to(np.eye(Lk, dtype=np.float32), (1, Hkv, Lk, Lk)).copy()   # values = one-hot rows
    out, _ = dec.decode_attention(q[None], k[None], eye)
    assert np.allclose(A, out[0], rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- paged storage
def test_rows_from_pages_inverts_a_scattering_into_pages():
    # catches: page and in-page index swapped, head and row axes swapped, a table read by physical page
    rng = np.random.default_rng(12)
    H, L, D, ps = 3, 37, 4, 8
    x = rng.standard_normal((H, L, D)).astype(np.float32)
    npages = 9
    table = rng.permutation(npages)[: (L + ps - 1) // ps]
    pages = np.full((npages, ps, H, D), np.nan, dtype=np.float32)
    for j in range(L):                                   # scatter by the definition of the layout
        for h in range(H):
            pages[table[j // ps], j % ps, h] = x[h, j]
    assert np.array_equal(orc.rows_from_pages(pages, table, L), x)
    ident = np.arange(npages)
    flat = pages.reshape(npages * ps, H, D)              # identity table: the view is a plain reshape
    assert np.array_equal(orc.rows_from_pages(pages, ident, L), np.transpose(flat[:L], (1, 0, 2)), equal_nan=True)

