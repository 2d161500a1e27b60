"""snapkv_compress_varlen: a batch of prompts of different lengths gets, prompt by prompt, exactly what
snapkv_compress gives (and so the oracle's result, checked on a sample), whatever the mix of lengths."""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload
from parity import check_against_oracle, run_gpu

pytestmark = pytest.mark.gpu


def prompts(lengths, **kw):
    base = dict(Hq=8, Hkv=4, D=128, W=32, pool_kind=0, p=7, C=256, dtype="bf16", clusters=(5, 5), radius=6)
    base.update(kw)
    return [Workload(f"vl_{i}_{L}", L=L, seed=900 + i, **base) for i, L in enumerate(lengths)]


def run_batch(snapkv, ws):
    cases = [workloads.generate(w, device="cuda") for w in ws]
    w0 = ws[0]
    oks = [torch.zeros((w0.Hkv, w0.C, w0.D), dtype=c["k"].dtype, device="cuda") for c in cases]
    ovs = [torch.zeros_like(t) for t in oks]
    ois = [torch.full((w0.Hkv, w0.C), -1, dtype=torch.int32, device="cuda") for _ in cases]
    kept = snapkv.snapkv_compress_varlen([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                         w0.pool_kind, w0.p, w0.C, oks, ovs, ois)
    torch.cuda.synchronize()
    return cases, oks, ovs, ois, kept


def compare_with_single_calls(snapkv, ws, cases, oks, ovs, ois, kept, oracle_on=()):
    for i, (w, c) in enumerate(zip(ws, cases)):
        ref = run_gpu(snapkv, c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C)
        rows = min(w.C, w.L)
        assert kept[i] == ref[4] == rows, (w.name, kept[i])
        assert np.array_equal(ois[i].cpu().numpy()[:, :rows], ref[3][:, :rows]), w.name
        assert torch.equal(oks[i][:, :rows], ref[1][:, :rows]) and torch.equal(ovs[i][:, :rows], ref[2][:, :rows]), w.name
        if i in oracle_on:
            check_against_oracle(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ref[0], oks[i], ovs[i],
                                 ois[i].cpu().numpy(), kept[i])


MIXES = {
    "ragged_mix": dict(lengths=[5003, 1301, 9000, 290, 2600]),                       # 290 fits the capacity: returned unchanged
    "gqa_avg_w16": dict(lengths=[4100, 12345, 800, 7001], Hq=16, Hkv=4, W=16, pool_kind=1, p=5, C=300),
    "equal_lengths": dict(lengths=[3000, 3000, 3000]),
    "one_long_many_short": dict(lengths=[40000, 600, 700, 650, 800, 620], C=512),    # most workgroups of the short heads are empty
    "d64_f16": dict(lengths=[2222, 5555, 3333], D=64, dtype="f16", C=200),
    "wide_window_runs_one_by_one": dict(lengths=[1500, 2100], W=160, C=320, p=5),
    "single_prompt": dict(lengths=[4321]),
}


@pytest.mark.parametrize("name", list(MIXES))
def test_batch_equals_single_calls(snapkv, name):
    kw = dict(MIXES[name])
    ws = prompts(kw.pop("lengths"), **kw)
    cases, oks, ovs, ois, kept = run_batch(snapkv, ws)
    compare_with_single_calls(snapkv, ws, cases, oks, ovs, ois, kept, oracle_on=(0, len(ws) - 1))
    assert snapkv.snapkv_sync_timeouts() == 0


def test_batch_larger_than_one_joint_launch(snapkv):
    """More prompts than one joint launch takes: split inside the call."""
    lengths = [600 + 37 * i for i in range(40)]
    ws = prompts(lengths, Hq=4, Hkv=2, C=128)
    cases, oks, ovs, ois, kept = run_batch(snapkv, ws)
    compare_with_single_calls(snapkv, ws, cases, oks, ovs, ois, kept)


def test_batch_back_to_back_with_single_calls(snapkv):
    """The batch and single calls share the library's scratch: neither may leave the other a stale state."""
    ws = prompts([5003, 1301, 2600])
    single = workloads.generate(ws[0], device="cuda")
    ref = run_gpu(snapkv, single["q_win"], single["k"], single["v"], ws[0].pool_kind, ws[0].p, ws[0].C)
    for _ in range(2):
        cases, oks, ovs, ois, kept = run_batch(snapkv, ws)
        assert np.array_equal(ois[0].cpu().numpy(), ref[3])
        again = run_gpu(snapkv, single["q_win"], single["k"], single["v"], ws[0].pool_kind, ws[0].p, ws[0].C)
        assert np.array_equal(again[3], ref[3]) and torch.equal(again[1], ref[1])
    assert snapkv.snapkv_sync_timeouts() == 0


def test_empty_batch_and_bad_prompt(snapkv):
    assert snapkv.snapkv_compress_varlen([], [], [], 0, 7, 64, [], [], []) == []
    ws = prompts([3000, 2000])
    cases = [workloads.generate(w, device="cuda") for w in ws]
    oks = [torch.zeros((4, 256, 128), dtype=torch.bfloat16, device="cuda") for _ in cases]
    ovs = [torch.zeros_like(t) for t in oks]
    ois = [torch.full((4, 256), -7, dtype=torch.int32, device="cuda") for _ in cases]
    with pytest.raises(snapkv.SnapKVError):      # an even pooling width: refused before anything is enqueued
        snapkv.snapkv_compress_varlen([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                      0, 6, 256, oks, ovs, ois)
    torch.cuda.synchronize()
    assert all(int(t.min()) == -7 and int(t.max()) == -7 for t in ois)


def test_batch_with_prompts_the_single_read_launch_does_not_hold(snapkv):
    """With the plans counting 16 resident workgroups the longer prompts of a batch are beyond the single-read
    launch: inside a batch they take two streaming passes (another rounding than the single call's path, so the
    reference is the oracle, prompt by prompt)."""
    snapkv.snapkv_set_scoring_scheme(4)
    try:
        ws = prompts([12000, 3000, 20000, 700], C=300)
        cases, oks, ovs, ois, kept = run_batch(snapkv, ws)
        for w, c, ok, ov, oi, kp in zip(ws, cases, oks, ovs, ois, kept):
            sc = torch.empty((w.Hkv, w.n), dtype=torch.float32, device="cuda")
            snapkv.snapkv_pooled_scores(c["q_win"], c["k"], w.pool_kind, w.p, sc)
            check_against_oracle(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, sc.cpu().numpy(), ok, ov,
                                 oi.cpu().numpy(), kp, own_topk_exact=False)
        assert snapkv.snapkv_sync_timeouts() == 0
    finally:
        snapkv.snapkv_set_scoring_scheme(0)
