"""snapkv_compress_static (the entry point for callers that cannot allocate: its scratch is a fixed array in
the library's device image) gives, bit for bit, what snapkv_compress_ws gives with a workspace of the
caller's: two calls in a row, the second on a smaller prompt, and a shape beyond the array is refused."""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload

pytestmark = pytest.mark.gpu


def both_ways(snapkv, w):
    c = workloads.generate(w, device="cuda")
    q, k, v = c["q_win"], c["k"], c["v"]
    outs = []
    for static in (True, False):
        ok = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
        ov = torch.zeros_like(ok)
        oi = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
        if static:
            kept = snapkv.snapkv_compress_static(q, k, v, w.pool_kind, w.p, w.C, ok, ov, oi)
        else:
            ws = torch.empty(snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W), dtype=torch.uint8, device="cuda")
            kept = snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, ok, ov, oi, workspace=ws)
        torch.cuda.synchronize()
        outs.append((kept, oi.cpu().numpy(), ok, ov))
    (ka, ia, oka, ova), (kb, ib, okb, ovb) = outs
    assert ka == kb == min(w.C, w.L)
    assert np.array_equal(ia, ib), f"{w.name}: kept positions differ"
    assert torch.equal(oka, okb) and torch.equal(ova, ovb), f"{w.name}: gathered rows differ"
    # the kept positions are sane in their own right: ascending, window last
    kc = w.C - w.W
    assert np.all(np.diff(ia, axis=1) > 0) and np.array_equal(ia[:, kc:], np.tile(np.arange(w.n, w.L), (w.Hkv, 1)))


def test_static_scratch_equals_caller_workspace_twice_in_a_row(snapkv):
    base = dict(Hq=8, Hkv=4, D=128, W=32, pool_kind=0, p=7, dtype="bf16", clusters=(6, 6), radius=6)
    first = Workload("static_first", L=9000, C=512, seed=7100, **base)
    second = Workload("static_second_smaller", L=2100, C=256, seed=7101, **base)
    assert snapkv.snapkv_workspace_bytes(first.L, first.Hq, first.Hkv, first.D, first.W) <= snapkv.STATIC_SCRATCH_BYTES
    both_ways(snapkv, first)
    both_ways(snapkv, second)      # finds the first call's contents in the array
    both_ways(snapkv, first)
    assert snapkv.snapkv_sync_timeouts() == 0


def test_static_scratch_refuses_shapes_beyond_the_array(snapkv):
    w = Workload("static_too_large", Hq=32, Hkv=32, D=128, L=131072, W=32, pool_kind=0, p=7, C=4096, dtype="bf16",
                 clusters=(1, 1), radius=1)
    assert snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W) > snapkv.STATIC_SCRATCH_BYTES
    # validation comes first: no tensor of that size is needed to see the refusal
    q = torch.zeros((w.Hq, w.W, w.D), dtype=torch.bfloat16, device="cuda")
    lib = snapkv.load()
    fake = q.data_ptr()
    rc = lib.snapkv_compress_static(0, fake, fake, fake, w.L, w.Hq, w.Hkv, w.D, w.W, 0, 7, w.C, fake, fake, fake, None)
    assert rc == -4 and snapkv.snapkv_strerror(rc) == "workspace missing or too small"
