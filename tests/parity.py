"""Shared checker for the GPU parity tests: HIP path vs the fp64 oracle on the same bytes."""
from __future__ import annotations

import numpy as np
import torch

from oracle import snapkv_oracle as orc
from paper_2404_14469_amd import workloads

REL_TOL = 1e-3        # pooled scores: |gpu - oracle| <= REL_TOL * |oracle| (spec tolerance)
ABS_FLOOR = 1e-30     # only excuses fp32 underflow of scores that are zero for every purpose


def run_gpu(pkg, q, k, v, pool_kind, p, C):
    """Calls the C ABI through the binding; returns host copies of everything it produced."""
    Hkv, L, D = k.shape
    W = q.shape[1]
    n = L - W
    scores = None
    if n > 0:
        sc = torch.full((Hkv, n), float("nan"), dtype=torch.float32, device=k.device)
        pkg.snapkv_pooled_scores(q, k, pool_kind, p, sc)
        scores = sc.cpu().numpy()
    out_k = torch.zeros((Hkv, C, D), dtype=k.dtype, device=k.device)
    out_v = torch.zeros((Hkv, C, D), dtype=k.dtype, device=k.device)
    out_idx = torch.full((Hkv, C), -1, dtype=torch.int32, device=k.device)
    kept = pkg.snapkv_compress(q, k, v, pool_kind, p, C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    return scores, out_k, out_v, out_idx.cpu().numpy(), kept


def check_against_oracle(q, k, v, pool_kind, p, C, scores, out_k, out_v, out_idx, kept, heads=None,
                         own_topk_exact=True, oracle_scores=None):
    """The parity bar, per KV head in `heads` (default: all).

    - pooled scores within REL_TOL relative of the oracle's;
    - kept positions: every position the oracle scores above T(1+tol) is kept, none below
      T(1-tol) is, T being the oracle's (C-W)-th largest score; inside the band either is right;
    - sharp self-consistency: the kept set is exactly the top-(C-W) of the GPU's own scores under
      (score descending, position ascending);
    - positions unique, ascending, window last; gathered K/V rows bit-identical to the inputs'.
    `oracle_scores` [Hkv, L-W] (fp64), when given, are the oracle's pooled scores computed beforehand (the
    plain-C oracle does a whole full-size layer at once); otherwise the numpy oracle is run head by head.
    Returns the number of band (near-tie) positions seen, for information.
    """
    Hkv, L, D = k.shape
    W = q.shape[1]
    n = L - W
    heads = list(range(Hkv)) if heads is None else list(heads)
    g = q.shape[0] // Hkv
    band_total = 0
    kb, vb = workloads.to_numpy_bits(k[heads]), workloads.to_numpy_bits(v[heads])
    okb, ovb = workloads.to_numpy_bits(out_k[heads]), workloads.to_numpy_bits(out_v[heads])
    if L <= C:
        assert kept == L
        for oi, hk in enumerate(heads):
            assert np.array_equal(out_idx[hk, :L], np.arange(L))
            assert np.array_equal(okb[oi, :L], kb[oi]) and np.array_equal(ovb[oi, :L], vb[oi])
        return 0
    assert kept == C
    kc = C - W
    qb = workloads.to_numpy_bits(q)
    for oi, hk in enumerate(heads):
        s_orc = (oracle_scores[hk] if oracle_scores is not None
                 else orc.pooled_scores(qb[hk * g:(hk + 1) * g], kb[oi:oi + 1], W, pool_kind, p)[0])
        s_gpu = scores[hk].astype(np.float64)
        assert np.all(np.isfinite(s_gpu)), f"head {hk}: non-finite GPU score"
        err = np.abs(s_gpu - s_orc)
        bad = err > REL_TOL * np.abs(s_orc) + ABS_FLOOR
        assert not bad.any(), (f"head {hk}: {bad.sum()} scores off; worst rel "
                               f"{(err / np.maximum(np.abs(s_orc), 1e-300)).max():.3e}")
        idx = out_idx[hk].astype(np.int64)
        assert np.all(np.diff(idx) > 0), f"head {hk}: positions not strictly ascending"
        assert idx[0] >= 0 and np.array_equal(idx[kc:], np.arange(n, L)), f"head {hk}: window rows"
        sel = idx[:kc]
        if kc > 0:
            assert sel[-1] < n
            T = np.sort(s_orc)[::-1][kc - 1]
            must_keep = np.nonzero(s_orc > T * (1 + REL_TOL))[0]
            must_drop = np.nonzero(s_orc < T * (1 - REL_TOL))[0]
            chosen = np.zeros(n, dtype=bool)
            chosen[sel] = True
            assert chosen[must_keep].all(), f"head {hk}: a clearly-above-threshold position was dropped"
            assert not chosen[must_drop].any(), f"head {hk}: a clearly-below-threshold position was kept"
            band_total += n - len(must_keep) - len(must_drop)
            # exact top-k of the GPU's own scores (float32 values, compared exactly); callers whose
            # `scores` come from a differently shaped launch than the kept set pass own_topk_exact=False
            if own_topk_exact:
                assert np.array_equal(sel, orc.select(scores[hk].astype(np.float64), kc)), \
                    f"head {hk}: kept set is not the exact top-k of the GPU's scores"
        assert np.array_equal(okb[oi], kb[oi][idx]), f"head {hk}: gathered K rows differ"
        assert np.array_equal(ovb[oi], vb[oi][idx]), f"head {hk}: gathered V rows differ"
    return band_total


def check_self_consistency(q, k, v, C, scores, out_k, out_v, out_idx, kept):
    """Size-independent properties on every head, computed without the oracle's arithmetic:
    positions unique/ascending/window-last, the kept set is the exact top-(C-W) of the GPU's own
    scores with ties to the lower position, and the gathered rows are the inputs' rows bit for bit
    (compared on the GPU with torch indexing)."""
    Hkv, L, D = k.shape
    W = q.shape[1]
    n = L - W
    assert kept == min(C, L)
    if L <= C:
        return
    kc = C - W
    idx_dev = torch.from_numpy(out_idx.astype(np.int64)).to(k.device)
    for hk in range(Hkv):
        idx = out_idx[hk].astype(np.int64)
        assert np.all(np.diff(idx) > 0) and idx[0] >= 0
        assert np.array_equal(idx[kc:], np.arange(n, L))
        if kc > 0:
            s = scores[hk]
            order = np.argsort(-s.astype(np.float64), kind="stable")[:kc]
            want = np.sort(order)
            if not np.array_equal(idx[:kc], want):
                extra = np.setdiff1d(idx[:kc], want)
                missing = np.setdiff1d(want, idx[:kc])
                raise AssertionError(
                    f"head {hk}: not the exact top-k of the GPU's scores: {len(extra)} kept beyond it "
                    f"(first {extra[:4].tolist()}, scores {s[extra[:4]].tolist()}), {len(missing)} missing "
                    f"(first {missing[:4].tolist()}, scores {s[missing[:4]].tolist()}), "
                    f"k-th score {float(np.sort(s)[::-1][kc - 1])!r}")
        assert torch.equal(out_k[hk].view(torch.uint8), k[hk][idx_dev[hk]].view(torch.uint8))
        assert torch.equal(out_v[hk].view(torch.uint8), v[hk][idx_dev[hk]].view(torch.uint8))


def gpu_vs_oracle(pkg, w, layer=0, heads=None, device="cuda"):
    case = workloads.generate(w, layer=layer, device=device)
    q, k, v = case["q_win"], case["k"], case["v"]
    res = run_gpu(pkg, q, k, v, w.pool_kind, w.p, w.C)
    band = check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, heads=heads)
    return case, res, band
