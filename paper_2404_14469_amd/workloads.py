"""Seeded synthetic prompt-phase Q/K/V for the SnapKV compression step.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no attention, softmax, pooling, selection or gathering), so both the HIP
path and the CPU oracle can be fed the same bytes from it without sharing
any code that computes the method.

The paper evaluates on LongBench-scale prompts (13K-32K tokens), on
needle-in-a-haystack style long contexts (131K-380K tokens) and on GQA
models (Sec. 5).  Those datasets and model weights are not available here;
the workloads below stand in for their *shapes* and for the structure the
method exploits: a few clusters of prefix keys that the observation-window
queries attend to (Sec. 3, Sec. 4.3) and, for the long-context case, one
single-token "needle" key deep in the prefix (Sec. 5.1.1).

Recipe (per call = one prompt, one layer):
  * Q_win [Hq, W, D], K [Hkv, L, D], V [Hkv, L, D] ~ N(0, 1) in fp32.
  * per KV head and cluster c: a random unit vector u_c and a centre drawn
    uniformly in the prefix [0, L-W); K rows within +-radius of the centre
    (clipped to the prefix) get += strength * u_c; every window query of every
    query head in that KV group gets += sum_c u_c.
  * optional needle: one prefix row of K gets += 3*sqrt(D)*u, every window
    query of the group gets += 4*u.
  * finally everything is rounded to the storage dtype (bf16, fp16 or fp32).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    Hq: int
    Hkv: int
    D: int
    L: int
    W: int
    pool_kind: int  # 0 = max, 1 = avg
    p: int
    C: int
    dtype: str  # "bf16" | "f16" | "f32"
    clusters: Tuple[int, int]  # (lo, hi) inclusive range of clusters per KV head
    radius: int
    strength: float = 3.0
    needle: bool = False
    layers: int = 1
    seed: int = 0

    @property
    def n(self) -> int:
        return self.L - self.W

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five named configurations.  Seeds are base seeds; layer l uses seed + l.
TINY = Workload("tiny", Hq=4, Hkv=4, D=64, L=512, W=32, pool_kind=0, p=7, C=128,
                dtype="f32", clusters=(4, 4), radius=4, seed=1001)
LLAMA2_7B_16K = Workload("llama2_7b_16k", Hq=32, Hkv=32, D=128, L=16384, W=32, pool_kind=0, p=7,
                         C=1024, dtype="bf16", clusters=(16, 16), radius=8, seed=1002)
MISTRAL_7B_GQA_32K = Workload("mistral_7b_gqa_32k", Hq=32, Hkv=8, D=128, L=32768, W=32, pool_kind=0,
                              p=7, C=2048, dtype="bf16", clusters=(16, 16), radius=8, layers=32,
                              seed=1003)
LONG_131K = Workload("long_131k", Hq=32, Hkv=32, D=128, L=131072, W=32, pool_kind=0, p=7, C=4096,
                     dtype="bf16", clusters=(32, 32), radius=8, needle=True, layers=32, seed=1004)
VARLEN_BASE = Workload("varlen", Hq=32, Hkv=8, D=128, L=0, W=16, pool_kind=1, p=5, C=1024,
                       dtype="bf16", clusters=(8, 32), radius=8, seed=1005)

CONFIGS: Dict[str, Workload] = {w.name: w for w in
                                (TINY, LLAMA2_7B_16K, MISTRAL_7B_GQA_32K, LONG_131K)}


def varlen_prompts(n_prompts: int = 8, lo: int = 4096, hi: int = 65536,
                   seed: int = VARLEN_BASE.seed) -> List[Workload]:
    """The batched-varlen configuration: lengths are drawn first, uniformly in [lo, hi]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    lens = torch.randint(lo, hi + 1, (n_prompts,), generator=g).tolist()
    return [VARLEN_BASE.with_(name=f"varlen_{i}", L=int(L), seed=seed + 1 + i)
            for i, L in enumerate(lens)]


def _unit(gen: torch.Generator, shape, device) -> torch.Tensor:
    u = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    return u / u.norm(dim=-1, keepdim=True)


def generate(w: Workload, layer: int = 0, device: str = "cpu") -> Dict[str, object]:
    """Draw one call's inputs.

    Returns a dict with torch tensors ``q_win`` [Hq, W, D], ``k`` and ``v`` [Hkv, L, D] in the
    workload's storage dtype on ``device``, plus the planted structure (``centres`` as a list
    per KV head, ``needle_pos`` per KV head or None) for sanity assertions.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + layer)
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed((w.seed + layer) * 7919 + 13)

    Hq, Hkv, D, L, W, n, g = w.Hq, w.Hkv, w.D, w.L, w.W, w.n, w.g
    q = torch.randn((Hq, W, D), generator=gen, device=dev, dtype=torch.float32)
    k = torch.randn((Hkv, L, D), generator=gen, device=dev, dtype=torch.float32)
    v = torch.randn((Hkv, L, D), generator=gen, device=dev, dtype=torch.float32)

    centres: List[List[int]] = []
    needle_pos: Optional[List[int]] = [] if w.needle else None
    lo, hi = w.clusters
    for hk in range(Hkv):
        nc = int(torch.randint(lo, hi + 1, (1,), generator=cpu_gen).item())
        cs = torch.randint(0, max(n, 1), (nc,), generator=cpu_gen).tolist() if n > 0 else []
        centres.append([int(c) for c in cs])
        if n <= 0:
            continue
        u = _unit(gen, (nc, D), dev)
        for ci, c in enumerate(cs):
            a, b = max(0, c - w.radius), min(n, c + w.radius + 1)
            k[hk, a:b, :] += w.strength * u[ci]
        q[hk * g:(hk + 1) * g, :, :] += u.sum(dim=0)
        if w.needle:
            pos = int(torch.randint(0, n, (1,), generator=cpu_gen).item())
            un = _unit(gen, (D,), dev)
            k[hk, pos, :] += 3.0 * math.sqrt(D) * un
            q[hk * g:(hk + 1) * g, :, :] += 4.0 * un
            needle_pos.append(pos)

    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.dtype]
    return {"q_win": q.to(tdt).contiguous(), "k": k.to(tdt).contiguous(),
            "v": v.to(tdt).contiguous(), "centres": centres, "needle_pos": needle_pos}


@dataclasses.dataclass(frozen=True)
class DecodeWorkload:
    """One decoding step over compacted caches: B sequences whose caches hold S valid rows of a
    capacity of cap (the kept prompt rows plus the tokens generated since)."""
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    S: int
    cap: int
    dtype: str = "bf16"
    ragged: bool = False   # per-sequence lengths drawn in [1, S] instead of S everywhere
    seed: int = 0


# Sec. 5.1.2 benchmarks decoding with the cache capped at 2048 prompt rows and 512 generated
# tokens on a 32-head, D=128 model at batch sizes 1 to 8: the last step attends to 2560 rows.
DECODE_CAPPED_B8 = DecodeWorkload("decode_capped_b8", B=8, Hq=32, Hkv=32, D=128, S=2560, cap=2560, seed=2001)
# The uncompressed cache of a 16K prompt at the batch size where the paper's baseline runs out of memory.
DECODE_FULL_16K_B2 = DecodeWorkload("decode_full_16k_b2", B=2, Hq=32, Hkv=32, D=128, S=16384 + 512,
                                    cap=16384 + 512, seed=2002)
# The capped cache at the same batch size, for the ratio between the two.
DECODE_CAPPED_B2 = DecodeWorkload("decode_capped_b2", B=2, Hq=32, Hkv=32, D=128, S=2560, cap=2560, seed=2003)
DECODE_CONFIGS: Dict[str, DecodeWorkload] = {w.name: w for w in (DECODE_CAPPED_B8, DECODE_FULL_16K_B2, DECODE_CAPPED_B2)}


def generate_decode(w: DecodeWorkload, device: str = "cpu") -> Dict[str, object]:
    """Draws q [B, Hq, D], k_cache and v_cache [B, Hkv, cap, D] ~ N(0, 1) and lens [B] int32 (or
    None).  A few cache rows per (sequence, KV head) get += 2 * u for a unit vector u that the
    queries of that group also get (+= 3 * u), so that the attention is peaked on a few rows as
    it is on a cache that kept the rows the queries look for.  Rows beyond a sequence's length
    hold large values that a correct result never sees."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed(w.seed * 7919 + 17)
    g = w.Hq // w.Hkv
    q = torch.randn((w.B, w.Hq, w.D), generator=gen, device=dev, dtype=torch.float32)
    k = torch.randn((w.B, w.Hkv, w.cap, w.D), generator=gen, device=dev, dtype=torch.float32)
    v = torch.randn((w.B, w.Hkv, w.cap, w.D), generator=gen, device=dev, dtype=torch.float32)
    lens = None
    if w.ragged:
        lens = torch.randint(1, w.S + 1, (w.B,), generator=cpu_gen, dtype=torch.int32)
        lens[0] = w.S
    u = _unit(gen, (w.B, w.Hkv, w.D), dev)
    for b in range(w.B):
        S = int(lens[b]) if lens is not None else w.S
        rows = torch.randint(0, S, (4,), generator=cpu_gen).tolist()
        for r in rows:
            k[b, :, r, :] += 2.0 * u[b]
        k[b, :, S:, :] = 1.0e4
        v[b, :, S:, :] = -3.0e4
    q += 3.0 * u.repeat_interleave(g, dim=1)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[w.dtype]
    return {"q": q.to(tdt).contiguous(), "k_cache": k.to(tdt).contiguous(), "v_cache": v.to(tdt).contiguous(),
            "lens": lens.to(dev) if lens is not None else None}


def to_numpy_bits(t: torch.Tensor):
    """Host copy of a tensor as a numpy array: fp32 as float32, fp16 as float16, bf16 as its uint16 bit
    patterns."""
    import numpy as np
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
