"""A bounded wait that gives up inside a kernel is reported, without a device synchronisation of the
library's: in the status word of snapkv_compress_ws_status, and one call late by the entries that use the
library's own scratch.  The condition is forced from the host with the test hook that bounds every wait
to zero polls; all kernels still run to their end and stay inside their buffers."""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload

pytestmark = pytest.mark.gpu

# several workgroups per head in the pooling + selection kernel: the first to reach a rendezvous has to wait
W = Workload("timeout", Hq=8, Hkv=4, D=128, L=9000, W=32, pool_kind=0, p=7, C=512, dtype="bf16", clusters=(6, 6),
             radius=6, seed=8100)


def buffers(k):
    ok = torch.zeros((W.Hkv, W.C, W.D), dtype=k.dtype, device="cuda")
    return ok, torch.zeros_like(ok), torch.full((W.Hkv, W.C), -1, dtype=torch.int32, device="cuda")


def test_status_word_reports_a_wait_that_gave_up(snapkv):
    c = workloads.generate(W, device="cuda")
    q, k, v = c["q_win"], c["k"], c["v"]
    ws = torch.empty(snapkv.snapkv_workspace_bytes(W.L, W.Hq, W.Hkv, W.D, W.W), dtype=torch.uint8, device="cuda")
    status = torch.full((1,), 12345, dtype=torch.int32, device="cuda")
    ok, ov, oi = buffers(k)
    assert snapkv.snapkv_compress_ws_status(q, k, v, W.pool_kind, W.p, W.C, ok, ov, oi, ws, status) == W.C
    torch.cuda.synchronize()
    assert int(status.item()) == W.C
    good = oi.cpu().numpy().copy()
    before = snapkv.snapkv_sync_timeouts()
    snapkv.snapkv_debug_set_wait_limit(0)
    try:
        ok2, ov2, oi2 = buffers(k)
        assert snapkv.snapkv_compress_ws_status(q, k, v, W.pool_kind, W.p, W.C, ok2, ov2, oi2, ws, status) == W.C
        torch.cuda.synchronize()
        gave_up = snapkv.snapkv_sync_timeouts() - before
    finally:
        snapkv.snapkv_debug_set_wait_limit(-2)     # the kernels' own bounds again, and the count back to zero
    assert int(status.item()) == snapkv.ERR_TIMEOUT
    assert gave_up > 0 and snapkv.snapkv_sync_timeouts() == 0
    # and the next call on the same workspace is sound again
    ok3, ov3, oi3 = buffers(k)
    assert snapkv.snapkv_compress_ws_status(q, k, v, W.pool_kind, W.p, W.C, ok3, ov3, oi3, ws, status) == W.C
    torch.cuda.synchronize()
    assert int(status.item()) == W.C
    assert np.array_equal(oi3.cpu().numpy(), good) and torch.equal(ok3, ok) and torch.equal(ov3, ov)


def test_own_scratch_entries_report_it_one_call_late(snapkv):
    c = workloads.generate(W, device="cuda")
    q, k, v = c["q_win"], c["k"], c["v"]
    ok, ov, oi = buffers(k)
    assert snapkv.snapkv_compress(q, k, v, W.pool_kind, W.p, W.C, ok, ov, oi) == W.C
    torch.cuda.synchronize()
    good = oi.cpu().numpy().copy()
    snapkv.snapkv_debug_set_wait_limit(0)
    try:
        ok2, ov2, oi2 = buffers(k)
        assert snapkv.snapkv_compress(q, k, v, W.pool_kind, W.p, W.C, ok2, ov2, oi2) == W.C   # enqueued: nothing known yet
        torch.cuda.synchronize()
    finally:
        snapkv.snapkv_debug_set_wait_limit(-2)
    with pytest.raises(snapkv.SnapKVError) as err:
        snapkv.snapkv_compress(q, k, v, W.pool_kind, W.p, W.C, ok2, ov2, oi2)
    assert err.value.code == snapkv.ERR_TIMEOUT
    ok3, ov3, oi3 = buffers(k)
    assert snapkv.snapkv_compress(q, k, v, W.pool_kind, W.p, W.C, ok3, ov3, oi3) == W.C     # said once
    torch.cuda.synchronize()
    assert np.array_equal(oi3.cpu().numpy(), good) and torch.equal(ok3, ok) and torch.equal(ov3, ov)
