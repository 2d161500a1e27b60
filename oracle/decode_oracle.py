"""fp64 CPU oracle for one decoding step of attention over a compacted KV cache.

TEST INFRASTRUCTURE ONLY.  Nothing in the product imports this file and it imports nothing
from the product; only tests, the smoke check and the bench's cpu_baseline leg call it.

After the prompt's KV cache has been compressed to C rows per head (Listing 1), every
generated token attends to those C rows plus the rows appended since (Sec. 5.1.2, "Decoding
Speed and Memory Bound": the cache stays at its capped size, so the cost of a step does not
grow with the prompt).  The operation has a plain definition, written out here in float64 on
the exact stored values:

    out[h, :] = sum_j softmax_j( q_h . k_j / sqrt(D) ) v_j ,   j over the S valid cache rows
    lse[h]    = log sum_j exp( q_h . k_j / sqrt(D) )           (natural logarithm)

with query head h reading KV head h // g (g = Hq / Hkv).  The new token sees every cached
row, its own included, so there is no mask beyond the valid length.  The 1/sqrt(D) scale is
the same standard one the scoring step uses.

Pins (tests/test_decode_oracle_pins.py): a zero query (mean of the value rows), one row
(that row), a dominant key, two keys against the logistic function written by hand,
invariance under a joint permutation of cache rows and under a common shift of all keys,
the head-group mapping, rows beyond the valid length being ignored, the merge law of two
cache segments through their lse, and scipy's softmax / logsumexp.  No function is unpinned.
"""
from __future__ import annotations

import numpy as np


def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 values of the stored ones: float arrays as is, uint16 as bf16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if x.dtype in (np.float16, np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def decode_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, lens=None):
    """q [B, Hq, D]; k_cache, v_cache [B, Hkv, cap, D]; lens: None (all cap rows valid), an int,
    or B ints (valid rows per sequence, 1 <= len <= cap).
    Returns (out [B, Hq, D], lse [B, Hq]) in float64."""
    q = widen(q)
    k_cache = widen(k_cache)
    v_cache = widen(v_cache)
    B, Hq, D = q.shape
    Bk, Hkv, cap, Dk = k_cache.shape
    if (Bk, Dk) != (B, D) or v_cache.shape != k_cache.shape or Hq % Hkv != 0:
        raise ValueError("shape mismatch")
    g = Hq // Hkv
    if lens is None:
        lens = [cap] * B
    elif np.ndim(lens) == 0:
        lens = [int(lens)] * B
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    for b in range(B):
        S = int(lens[b])
        if S < 1 or S > cap:
            raise ValueError("valid length out of range")
        for h in range(Hq):
            kh = k_cache[b, h // g, :S]
            vh = v_cache[b, h // g, :S]
            s = kh @ q[b, h] / np.sqrt(float(D))
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[b, h] = (e / z) @ vh
            lse[b, h] = m + np.log(z)
    return out, lse
