"""fp64 CPU oracle for the SnapKV prompt-KV compression step (arXiv 2404.14469).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is
checked against.  Nothing in the product imports it; it imports nothing from the
product.  Only tests, the smoke check and the bench's cpu_baseline leg call it.

SnapKV is a heuristic defined by its procedure (Sec. 4.1, Listing 1; Eq. 1-2), so the
oracle is that procedure, step by step, in the paper's order, in float64 on the exact
input values (bf16 / fp32 widened exactly):

  1. logits  s[i, j] = q_i . k_j / sqrt(D) for the last W prompt queries against all L
     keys (Listing 1, the compute_attn call; the scale is the standard one - the paper
     leaves compute_attn undefined).
  2. prompt-phase causal mask: window query i sits at position n + i (n = L - W), so key
     j is hidden when j > n + i.  Only the trailing W x W block is affected.
  3. row softmax over all L keys ("softmax-normalized attention features", Sec. 4).
  4. vote[j] = sum over the W window rows, prefix columns j < n only (Eq. 1; the upper
     limit printed there would give W+1 terms, Listing 1 sums exactly the W rows).
  5. 1-D pooling with kernel p, stride 1, padding p//2 (Sec. 4.3, Listing 1): max pooling
     ignores positions outside [0, n); average pooling pads with zeros and always divides
     by p.  Pooling never sees window columns (they are sliced off before it).
  6. GQA (the paper's listing has equal head counts): pooled votes are summed over the
     g = Hq/Hkv query heads of a KV group *after* pooling; selection is per KV head.
  7. top-(C - W) positions per head (Eq. 2 / Listing 1), ties broken to the lower index,
     emitted in ascending position order.
  8. kept rows = selected prefix rows followed by the W window rows (Listing 1, the two
     gathers and concatenations).
  9. short prompts (L <= C) are returned unchanged (Listing 1, the first branch).

A second form takes the window rows' log-sum-exp as an input (window_lse / window_probs_given_lse;
pooled_scores and compress with lse=...): the quantity a block-wise attention prefill already
holds for every query row (Sec. 4.1 runs the step at the end of prompt encoding), which makes
step 3 a single exponential.  It is pinned to a hand-worked two-key case, to a library
log-sum-exp over the visible keys, to the softmax path (true lse changes nothing) and to the
row-scaling law of an offset lse.

A third form, compress_per_query_head, keeps one cache per query head of a grouped-query model
(the listing's equal head counts, reached by repeating KV heads); it is pinned to single-head
problems solved one by one, to the grouped form at g = 1 and to planted keys that only one query
head of a group looks for.

The hit rate of Sec. 4 (Eq. 3-7; current_attention, hit_rate_counts, hit_rate) is a quality probe:
how many of the positions the generated token attends to above a threshold the voting had kept.
Pinned to a uniform field (zero query), to planted keys with a hand-counted overlap and to a loop
over Python sets on tiny inputs.

Pins (tests/test_oracle_*.py): closed forms for all-zero queries (harmonic numbers, both
pool kinds and the tie rule), softmax rows summing to one, mass conservation, shift
invariance, permutation equivariance, nested selections, the W=1/p=1 special case against
a plain sort of raw logits, a planted one-hot key, torch-CPU library routines for the MHA
case, a pure-Python loop enumeration on tiny inputs and an independently written plain-C
version (oracle/snapkv_oracle.c).  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np

POOL_MAX = 0
POOL_AVG = 1


def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 view of the stored values: float arrays (IEEE half, single, double) as is,
    uint16 as bf16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if x.dtype in (np.float16, np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def window_probs(q_h: np.ndarray, k_h: np.ndarray) -> np.ndarray:
    """Steps 1-3 for one query head: P[W, L], each row a softmax over the keys it may see."""
    q = widen(q_h)
    k = widen(k_h)
    W, D = q.shape
    L = k.shape[0]
    n = L - W
    s = (q @ k.T) / np.sqrt(np.float64(D))                      # step 1
    j = np.arange(L)[None, :]
    i = np.arange(W)[:, None]
    s = np.where(j > n + i, -np.inf, s)                         # step 2
    s = s - s.max(axis=1, keepdims=True)                        # step 3
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def vote(P: np.ndarray) -> np.ndarray:
    """Step 4: column sum over the window rows, prefix columns only."""
    W, L = P.shape
    return P[:, :L - W].sum(axis=0)


def pool1d(x: np.ndarray, pool_kind: int, p: int) -> np.ndarray:
    """Step 5: stride-1 pooling with padding p//2 over a 1-D score vector."""
    if p < 1 or p % 2 == 0:
        raise ValueError("pool kernel must be odd and >= 1")
    n = x.shape[0]
    r = p // 2
    out = np.empty(n, dtype=np.float64)
    for jj in range(n):
        lo, hi = max(0, jj - r), min(n - 1, jj + r)
        seg = x[lo:hi + 1]
        if pool_kind == POOL_MAX:
            out[jj] = seg.max()
        elif pool_kind == POOL_AVG:
            out[jj] = seg.sum() / p
        else:
            raise ValueError("pool_kind must be 0 (max) or 1 (avg)")
    return out


def _pool1d_fast(x: np.ndarray, pool_kind: int, p: int) -> np.ndarray:
    """Same values as pool1d, vectorised so that 131072-long rows finish quickly.

    Max: out-of-range taps are -inf (bitwise equal to pool1d).  Avg: out-of-range taps are 0;
    the order in which the p taps are added may differ from pool1d's, so tests compare the
    two to 1e-14 relative rather than bitwise.
    """
    n = x.shape[0]
    r = p // 2
    pad = -np.inf if pool_kind == POOL_MAX else 0.0
    xp = np.concatenate([np.full(r, pad), x, np.full(r, pad)])
    taps = np.stack([xp[t:t + n] for t in range(p)], axis=0)
    if pool_kind == POOL_MAX:
        return taps.max(axis=0)
    if pool_kind == POOL_AVG:
        return taps.sum(axis=0) / p
    raise ValueError("pool_kind must be 0 (max) or 1 (avg)")


def window_lse(q_h: np.ndarray, k_h: np.ndarray) -> np.ndarray:
    """Natural log of each window row's softmax denominator, lse[i] = log sum_j exp(s[i, j]) over the
    keys row i may see (steps 1-2, then the logarithm of step 3's normaliser).  This is the quantity
    an attention prefill that works block by block keeps per query row."""
    q = widen(q_h)
    k = widen(k_h)
    W, D = q.shape
    L = k.shape[0]
    n = L - W
    s = (q @ k.T) / np.sqrt(np.float64(D))
    j = np.arange(L)[None, :]
    i = np.arange(W)[:, None]
    s = np.where(j > n + i, -np.inf, s)
    m = s.max(axis=1)
    return m + np.log(np.exp(s - m[:, None]).sum(axis=1))


def window_probs_given_lse(q_h: np.ndarray, k_h: np.ndarray, lse_h: np.ndarray) -> np.ndarray:
    """Steps 1-3 when the rows' log-sum-exp is handed in instead of computed: P = exp(s - lse),
    masked keys 0.  With lse = window_lse(q_h, k_h) this is window_probs(q_h, k_h); any other lse
    scales row i by exp(true_lse[i] - lse[i])."""
    q = widen(q_h)
    k = widen(k_h)
    W, D = q.shape
    L = k.shape[0]
    n = L - W
    s = (q @ k.T) / np.sqrt(np.float64(D))
    j = np.arange(L)[None, :]
    i = np.arange(W)[:, None]
    s = np.where(j > n + i, -np.inf, s)
    return np.exp(s - np.asarray(lse_h, dtype=np.float64)[:, None])


def pooled_scores(q_win: np.ndarray, k: np.ndarray, W: int, pool_kind: int, p: int,
                  kv_heads=None, lse=None) -> np.ndarray:
    """Steps 1-6: score[Hkv, n] (or only the listed KV heads, in the order given).  With lse
    [Hq, W] the softmax denominators are taken from it (window_probs_given_lse)."""
    Hq = q_win.shape[0]
    Hkv, L, _ = k.shape
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    if q_win.shape[1] != W or W < 1 or W > L:
        raise ValueError("bad window")
    if p < 1 or p % 2 == 0:
        raise ValueError("pool kernel must be odd and >= 1")
    g = Hq // Hkv
    n = L - W
    heads = range(Hkv) if kv_heads is None else list(kv_heads)
    out = np.zeros((len(heads), n), dtype=np.float64)
    for oi, hk in enumerate(heads):
        for h in range(hk * g, (hk + 1) * g):
            P = window_probs(q_win[h], k[hk]) if lse is None else window_probs_given_lse(q_win[h], k[hk], lse[h])
            v_h = vote(P)
            out[oi] += _pool1d_fast(v_h, pool_kind, p)              # step 6: pool, then group sum
    return out


def select(score: np.ndarray, kcount: int) -> np.ndarray:
    """Step 7: the kcount best positions under (score descending, index ascending), ascending."""
    n = score.shape[0]
    if kcount < 0 or kcount > n:
        raise ValueError("kcount out of range")
    order = np.argsort(-score, kind="stable")       # stable: equal scores stay in index order
    return np.sort(order[:kcount]).astype(np.int64)


def compress(q_win: np.ndarray, k: np.ndarray, v: np.ndarray, W: int, pool_kind: int, p: int,
             C: int, kv_heads=None, lse=None):
    """The whole step.  Returns (out_k, out_v, out_idx, kept, score).

    out_k/out_v are [H, kept, D] in the *storage* dtype of k/v (rows copied, never recomputed),
    out_idx is [H, kept] int64, kept = min(C, L), score is [H, n] float64 (None on bypass).
    """
    Hkv, L, D = k.shape
    if v.shape != k.shape:
        raise ValueError("k and v must have the same shape")
    if W > C:
        raise ValueError("window larger than capacity")
    heads = list(range(Hkv)) if kv_heads is None else list(kv_heads)
    if L <= C:                                                     # step 9
        idx = np.tile(np.arange(L, dtype=np.int64), (len(heads), 1))
        return k[heads].copy(), v[heads].copy(), idx, L, None
    n = L - W
    score = pooled_scores(q_win, k, W, pool_kind, p, kv_heads=heads, lse=lse)
    out_idx = np.empty((len(heads), C), dtype=np.int64)
    out_k = np.empty((len(heads), C, D), dtype=k.dtype)
    out_v = np.empty((len(heads), C, D), dtype=v.dtype)
    for oi, hk in enumerate(heads):
        sel = select(score[oi], C - W)                             # step 7
        idx = np.concatenate([sel, np.arange(n, L, dtype=np.int64)])   # step 8
        out_idx[oi] = idx
        out_k[oi] = k[hk][idx]
        out_v[oi] = v[hk][idx]
    return out_k, out_v, out_idx, C, score


def compress_per_query_head(q_win: np.ndarray, k: np.ndarray, v: np.ndarray, W: int, pool_kind: int,
                            p: int, C: int):
    """The step as Listing 1 states it, with one cache per *query* head: the listing's tensors have
    equal head counts, which a grouped-query model reaches by repeating every KV head for the g
    query heads that read it (query head h reads KV head h // g).  Each query head then votes,
    pools and selects alone (no sum over the group, cf. step 6) and gets its own C kept rows.
    Returns (out_k [Hq, kept, D], out_v, out_idx [Hq, kept], kept, score [Hq, n])."""
    Hq = q_win.shape[0]
    Hkv = k.shape[0]
    if Hq % Hkv != 0:
        raise ValueError("Hq must be a multiple of Hkv")
    g = Hq // Hkv
    return compress(q_win, np.repeat(k, g, axis=0), np.repeat(v, g, axis=0), W, pool_kind, p, C)


def capacity_for_rate(L: int, W: int, rate: float) -> int:
    """Capacity C = W + k for the rate form of Sec. 4 ("Voting"): k = floor(rate * L_prefix) prefix
    positions are kept, L_prefix = L - W.  The product is taken in IEEE double, as printed (no
    rational arithmetic): 0.29 * 100 is 28.999999999999996 and gives 28."""
    if not (0.0 <= rate <= 1.0) or W < 1 or W > L:
        raise ValueError("rate must be in [0, 1] and 1 <= W <= L")
    import math
    return W + int(math.floor(float(rate) * float(L - W)))


def current_attention(q_cur: np.ndarray, k: np.ndarray) -> np.ndarray:
    """A_cur of Sec. 4 ("Hit Rate") before it is cut to the prefix: the softmax-normalised attention
    of the query of the token being generated, q_cur [Hq, D], over all Lk keys it sees, k [Hkv, Lk, D]
    (query head h reads KV head h // g; scale 1/sqrt(D) as everywhere).  Returns [Hq, Lk] float64."""
    q_cur = widen(q_cur)
    k = widen(k)
    Hq, D = q_cur.shape
    Hkv = k.shape[0]
    g = Hq // Hkv
    A = np.empty((Hq, k.shape[1]), dtype=np.float64)
    for h in range(Hq):
        s = k[h // g] @ q_cur[h] / np.sqrt(float(D))
        e = np.exp(s - s.max())
        A[h] = e / e.sum()
    return A


def hit_rate_counts(A_cur: np.ndarray, idx: np.ndarray, theta: float):
    """Eq. 3-7 as counts.  A_cur [Hq, n]: current attention over the n prefix positions; idx
    [Hidx, kc]: the prefix positions voting selected, per KV head (Hidx = Hkv: query head h is checked
    against the selection of its KV head) or per query head (Hidx = Hq).  Per query head:
    important = number of positions with A_cur > theta (the threshold mask), hits = number of those
    that are selected (the overlap O).  The hit rate is H = sum(hits) / sum(important)."""
    Hq, n = A_cur.shape
    Hidx = idx.shape[0]
    div = Hq // Hidx
    M_vote = np.zeros((Hq, n), dtype=bool)
    for h in range(Hq):
        M_vote[h, idx[h // div]] = True
    M_thr = A_cur > theta
    O = np.logical_and(M_thr, M_vote)
    return M_thr.sum(axis=1).astype(np.int64), O.sum(axis=1).astype(np.int64)


def hit_rate(important: np.ndarray, hits: np.ndarray) -> float:
    """H of Eq. 7 from the counts; nan when nothing is above the threshold."""
    tot = int(np.sum(important))
    return float(np.sum(hits)) / tot if tot > 0 else float("nan")


def rows_from_pages(pages: np.ndarray, block_table: np.ndarray, L: int) -> np.ndarray:
    """Logical [H, L, D] view of a paged cache: pages [num_pages, page_size, H, D] (the rows of a page
    are token-major), block_table[i] = physical page of logical page i.  Listing 1 indexes K and V by
    (head, position) whatever their storage, so the step on a paged cache is the step on this view."""
    num_pages, ps, H, D = pages.shape
    out = np.empty((H, L, D), dtype=pages.dtype)
    for j in range(L):
        out[:, j, :] = pages[int(block_table[j // ps]), j % ps]
    return out

