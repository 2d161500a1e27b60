"""CPU-only checks of the boundary: the library loads, exports what the header declares, and its
host-side argument validation returns the documented codes before any GPU work (no compute)."""
import ctypes
import os
import re

import pytest

import paper_2404_14469_amd as pkg
from paper_2404_14469_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # non-null, 16-byte aligned, never dereferenced: validation fails first
ODD = 0x1008           # 8-byte aligned only


def header_symbols():
    text = open(os.path.join(ROOT, "include", "snapkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(snapkv_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pkg.load()
    names = header_symbols()
    assert set(names) == set(pkg.SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_strerror():
    assert pkg.snapkv_version() >= 100
    assert pkg.snapkv_strerror(-1) == "invalid argument"
    assert pkg.snapkv_strerror(-4) == "workspace missing or too small"
    assert pkg.snapkv_strerror(-99) == "unknown error"


def compress_code(**kw):
    a = dict(q=FAKE, k=FAKE, v=FAKE, L=4096, Hq=8, Hkv=8, D=128, W=32, kind=0, p=7, C=512,
             ok=FAKE, ov=FAKE, oi=FAKE)
    a.update(kw)
    return pkg.load().snapkv_compress(a["q"], a["k"], a["v"], a["L"], a["Hq"], a["Hkv"], a["D"], a["W"],
                                      a["kind"], a["p"], a["C"], a["ok"], a["ov"], a["oi"], None)


@pytest.mark.parametrize("kw,code", [
    (dict(q=None), -1), (dict(k=None), -1), (dict(v=None), -1), (dict(ok=None), -1),
    (dict(ov=None), -1), (dict(oi=None), -1),
    (dict(L=0), -1), (dict(W=0), -1), (dict(W=5000), -1), (dict(W=64, C=32), -1),
    (dict(p=4), -1), (dict(p=0), -1), (dict(p=-3), -1), (dict(kind=2), -1), (dict(Hq=12, Hkv=8), -1),
    (dict(Hkv=0), -1), (dict(C=0), -1),
    (dict(D=96), -2), (dict(D=256), -2), (dict(p=131), -2), (dict(L=2**31), -2), (dict(L=2**24 + 33), -2),
    (dict(q=ODD), -3), (dict(k=ODD), -3), (dict(v=ODD), -3), (dict(ok=ODD), -3), (dict(ov=ODD), -3),
    (dict(oi=0x1002), -3),
])
def test_compress_rejects_bad_arguments_on_the_host(kw, code):
    assert compress_code(**kw) == code


def test_scores_and_select_reject_bad_arguments():
    lib = pkg.load()
    assert lib.snapkv_pooled_scores(FAKE, FAKE, 4096, 8, 8, 128, 32, 0, 7, None, None) == -1
    assert lib.snapkv_pooled_scores(FAKE, FAKE, 4096, 8, 8, 128, 32, 0, 6, FAKE, None) == -1
    assert lib.snapkv_pooled_scores_f32(FAKE, FAKE, 4096, 8, 8, 100, 32, 0, 7, FAKE, None) == -2
    assert lib.snapkv_pooled_scores(FAKE, FAKE, 32, 8, 8, 128, 32, 0, 7, FAKE, None) == 0   # empty prefix
    # handed-in log-sum-exp: missing, misaligned, bad dtype code, too many window rows per query head
    lse_args = (4096, 8, 8, 128, 32, 0, 7)
    assert lib.snapkv_pooled_scores_lse(0, FAKE, FAKE, None, *lse_args, FAKE, None) == -1
    assert lib.snapkv_pooled_scores_lse(0, FAKE, FAKE, FAKE + 2, *lse_args, FAKE, None) == -3
    assert lib.snapkv_pooled_scores_lse(5, FAKE, FAKE, FAKE, *lse_args, FAKE, None) == -1
    assert lib.snapkv_pooled_scores_f16(FAKE, FAKE, 4096, 8, 8, 96, 32, 0, 7, FAKE, None) == -2
    assert lib.snapkv_compress_lse(0, FAKE, FAKE, FAKE, None, *lse_args, 512, FAKE, FAKE, FAKE, None) == -1
    assert lib.snapkv_compress_lse(0, FAKE, FAKE, FAKE, FAKE, 4096, 8, 8, 128, 32, 0, 6, 512, FAKE, FAKE, FAKE, None) == -1
    # strided K / V: row stride below D, negative head stride, strides that break 16-byte alignment
    st_args = lambda khs, krs, vhs, vrs: (0, FAKE, FAKE, FAKE, 4096, 8, 8, 128, 32, khs, krs, vhs, vrs, 0, 7, 512,
                                          FAKE, FAKE, FAKE, None)
    assert lib.snapkv_compress_strided(*st_args(4096 * 128, 64, 4096 * 128, 128)) == -1
    assert lib.snapkv_compress_strided(*st_args(-128, 128, 4096 * 128, 128)) == -1
    assert lib.snapkv_compress_strided(*st_args(4096 * 128, 132, 4096 * 128, 128)) == -3
    assert lib.snapkv_compress_strided(*st_args(128, 8 * 128, 4096 * 128 + 4, 128)) == -3
    assert lib.snapkv_select_topk(None, 1, 10, 2, FAKE, None) == -1
    assert lib.snapkv_select_topk(FAKE, 1, 10, 11, FAKE, None) == -1
    assert lib.snapkv_select_topk(FAKE, 1, 10, 0, FAKE, None) == 0
    assert lib.snapkv_compress_ws(7, FAKE, FAKE, FAKE, 4096, 8, 8, 128, 32, 0, 7, 512, FAKE, FAKE, FAKE,
                                  FAKE, 1 << 30, None) == -1
    # explicit workspace: missing, too small, misaligned
    need = pkg.snapkv_workspace_bytes(4096, 8, 8, 128, 32)
    args = (0, FAKE, FAKE, FAKE, 4096, 8, 8, 128, 32, 0, 7, 512, FAKE, FAKE, FAKE)
    assert lib.snapkv_compress_ws(*args, None, need, None) == -4
    assert lib.snapkv_compress_ws(*args, 0x10000, need - 1, None) == -4
    assert lib.snapkv_compress_ws(*args, 0x10010, need, None) == -3


def test_capacity_for_rate_matches_the_oracle():
    """Host arithmetic, so it runs without a GPU: both sides floor the same IEEE-double product."""
    import random
    from oracle import snapkv_oracle as orc
    rnd = random.Random(5)
    cases = [(100 + 32, 32, 0.29), (1000, 32, 0.0), (1000, 32, 1.0), (35, 32, 0.999), (131072, 32, 0.03125)]
    cases += [(rnd.randint(40, 200000), rnd.choice([1, 16, 32, 64]), rnd.random()) for _ in range(200)]
    for L, W, rate in cases:
        assert pkg.snapkv_capacity_for_rate(L, W, rate) == orc.capacity_for_rate(L, W, rate), (L, W, rate)
    assert pkg.snapkv_capacity_for_rate(132, 32, 0.29) == 32 + 28      # 0.29 * 100 is just under 29 in double
    for bad in ((100, 32, -0.1), (100, 32, 1.01), (100, 0, 0.5), (10, 32, 0.5), (100, 32, float("nan"))):
        with pytest.raises(pkg.SnapKVError):
            pkg.snapkv_capacity_for_rate(*bad)


def test_workspace_bytes():
    assert pkg.snapkv_workspace_bytes(0, 8, 8, 128, 32) == 0
    assert pkg.snapkv_workspace_bytes(4096, 8, 3, 128, 32) == 0
    assert pkg.snapkv_workspace_bytes(4096, 8, 8, 96, 32) == 0
    a = pkg.snapkv_workspace_bytes(4096, 8, 8, 128, 32)
    b = pkg.snapkv_workspace_bytes(8192, 8, 8, 128, 32)
    assert 0 < a < b and a % 256 == 0
    # must at least hold the votes and the pooled scores
    assert a >= 2 * 8 * (4096 - 32) * 4


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros((2, 4, 64), dtype=torch.bfloat16)
    k = torch.zeros((2, 64, 64), dtype=torch.bfloat16)
    out = torch.zeros((2, 16, 64), dtype=torch.bfloat16)
    idx = torch.zeros((2, 16), dtype=torch.int32)
    with pytest.raises(ValueError):
        pkg.snapkv_compress(q, k, k, 0, 3, 16, out, out.clone(), idx, stream=0)


def test_workload_generator_shapes_and_determinism():
    import torch
    w = workloads.TINY
    a = workloads.generate(w)
    b = workloads.generate(w)
    assert a["q_win"].shape == (4, 32, 64) and a["k"].shape == (4, 512, 64)
    assert a["k"].dtype == torch.float32
    assert torch.equal(a["k"], b["k"]) and torch.equal(a["q_win"], b["q_win"])
    c = workloads.generate(w, layer=1)
    assert not torch.equal(a["k"], c["k"])
    w2 = w.with_(dtype="bf16", needle=True)
    d = workloads.generate(w2)
    assert d["k"].dtype == torch.bfloat16 and len(d["needle_pos"]) == 4
    bits = workloads.to_numpy_bits(d["k"])
    assert bits.dtype.name == "uint16" and bits.shape == (4, 512, 64)
    lens = [p.L for p in workloads.varlen_prompts()]
    assert len(lens) == 8 and all(4096 <= x <= 65536 for x in lens)
    assert lens == [p.L for p in workloads.varlen_prompts()]
