"""GPU parity of snapkv_hit_rate (through the C ABI) against the oracle's Eq. 3-7 counts.

The counts are integers, but whether a position counts depends on A_cur > theta, which the GPU decides
in fp32 and the oracle in fp64.  A_cur on the GPU is accurate to well under 1e-3 relative (fp32 logits and
log-sum-exp), so the test brackets every count between the oracle's counts at theta*(1+1e-3) and
theta*(1-1e-3); where no A_cur lies in that band the bracket is a single value and the match is exact.
"""
import numpy as np
import pytest
import torch

from oracle import snapkv_oracle as orc
from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload

pytestmark = pytest.mark.gpu

TOL = 1e-3


def small(name, **kw):
    base = dict(Hq=8, Hkv=4, D=128, L=3000, W=32, pool_kind=0, p=7, C=256, dtype="bf16",
                clusters=(6, 6), radius=5, seed=50)
    base.update(kw)
    return Workload(name, **base)


def run_case(snapkv, w, theta, per_query_head=False):
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    hout = w.Hq if per_query_head else w.Hkv
    out_k = torch.empty((hout, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.empty_like(out_k)
    out_idx = torch.empty((hout, w.C), dtype=torch.int32, device="cuda")
    fn = snapkv.snapkv_compress_per_query_head if per_query_head else snapkv.snapkv_compress
    fn(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    q_cur = q[:, -1, :].contiguous()          # the last prompt query stands in for the first generated one
    counts = torch.full((w.Hq, 2), -1, dtype=torch.int32, device="cuda")
    snapkv.snapkv_hit_rate(q_cur, k, w.n, out_idx, w.C - w.W, theta, counts)
    torch.cuda.synchronize()
    A = orc.current_attention(workloads.to_numpy_bits(q_cur), workloads.to_numpy_bits(k))[:, :w.n]
    idx = out_idx.cpu().numpy()[:, :w.C - w.W].astype(np.int64)
    return counts.cpu().numpy(), A, idx


def check(counts, A, idx, theta):
    imp_lo, hit_lo = orc.hit_rate_counts(A, idx, theta * (1 + TOL))
    imp_hi, hit_hi = orc.hit_rate_counts(A, idx, theta * (1 - TOL))
    assert np.all(imp_lo <= counts[:, 0]) and np.all(counts[:, 0] <= imp_hi), (counts[:, 0], imp_lo, imp_hi)
    assert np.all(hit_lo <= counts[:, 1]) and np.all(counts[:, 1] <= hit_hi), (counts[:, 1], hit_lo, hit_hi)
    return int((imp_hi - imp_lo).sum())


CASES = [
    (small("hr_gqa"), 1e-3),
    (small("hr_gqa_low_theta"), 1e-4),
    (small("hr_mha_ragged", Hq=4, Hkv=4, L=2777, C=200), 5e-4),
    (small("hr_d64_w16", Hq=16, Hkv=2, D=64, W=16, L=5000, C=512, pool_kind=1, p=5), 2e-4),
    (small("hr_long", Hq=4, Hkv=2, L=70000, C=1024, clusters=(12, 12)), 1e-4),      # several counting chunks
    (small("hr_f16", dtype="f16", L=2100), 1e-3),
    (small("hr_tiny", Hq=2, Hkv=1, L=40, W=8, C=16, clusters=(1, 1), radius=2), 1e-2),
]


@pytest.mark.parametrize("w,theta", CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_hit_rate_counts_match_oracle(snapkv, w, theta):
    counts, A, idx = run_case(snapkv, w, theta)
    check(counts, A, idx, theta)
    assert counts[:, 0].sum() > 0                      # the threshold picks something on these inputs
    assert np.all(counts[:, 1] <= counts[:, 0]) and np.all(counts[:, 1] <= idx.shape[1])


def test_hit_rate_with_one_selection_per_query_head(snapkv):
    w = small("hr_pqh", Hq=8, Hkv=2)
    counts, A, idx = run_case(snapkv, w, 1e-3, per_query_head=True)
    assert idx.shape[0] == w.Hq
    check(counts, A, idx, 1e-3)


def test_hit_rate_exact_on_planted_keys(snapkv):
    """Attention concentrated on a few planted keys, threshold far from every value: exact counts."""
    Hq, Hkv, L, D, n = 4, 2, 600, 128, 560
    g = torch.Generator().manual_seed(3)
    k = (torch.randn((Hkv, L, D), generator=g) * 0.05)
    q = torch.zeros((Hq, D))
    planted = {0: [5, 100, 559], 1: [7], 2: [300, 301], 3: [580]}      # 580 lies outside the prefix
    for h, rows in planted.items():
        u = torch.zeros(D)
        u[h] = 1.0
        q[h] = 40.0 * u
        for r in rows:
            k[h // 2, r] += 8.0 * u
    qd, kd = q.to(torch.bfloat16).cuda(), k.to(torch.bfloat16).cuda()
    idx = torch.tensor([[5, 100, 200, 300], [7, 300, 400, 500]], dtype=torch.int32, device="cuda")
    counts = torch.empty((Hq, 2), dtype=torch.int32, device="cuda")
    snapkv.snapkv_hit_rate(qd, kd, n, idx, 4, 0.05, counts)
    torch.cuda.synchronize()
    A = orc.current_attention(workloads.to_numpy_bits(qd), workloads.to_numpy_bits(kd))[:, :n]
    imp, hits = orc.hit_rate_counts(A, idx.cpu().numpy().astype(np.int64), 0.05)
    assert imp.tolist() == [3, 1, 2, 0] and hits.tolist() == [2, 0, 1, 0]     # hand-counted
    assert counts.cpu().numpy().tolist() == [[3, 2], [1, 0], [2, 1], [0, 0]]
    assert orc.hit_rate(imp, hits) == 0.5


def test_hit_rate_rejects_bad_arguments(snapkv):
    q = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((2, 100, 128), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((2, 8), dtype=torch.int32, device="cuda")
    counts = torch.empty((4, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_hit_rate(q, k, 101, idx, 4, 0.1, counts)              # n > Lk
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_hit_rate(q, k, 50, idx, 9, 0.1, counts)               # kcount > stride
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_hit_rate(q, k, 50, idx[:, :6].contiguous().view(3, 4), 2, 0.1, counts)   # 3 rows do not divide 4 heads
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_hit_rate(q.float(), k.float(), 50, idx, 4, 0.1, counts)                  # fp32 storage
