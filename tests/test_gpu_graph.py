"""The compression step and the decoding step recorded into a HIP graph and replayed.

Callers with launch-bound inner loops capture the calls once and replay them.  The entry point with a
caller-provided workspace allocates nothing and clears its scratch with a fill kernel (no memset
nodes), so it can be captured; each replay is checked against an eager call on the same inputs, with
eager work and synchronisations between the replays.
"""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import DecodeWorkload, Workload

pytestmark = pytest.mark.gpu


def test_compress_ws_replays_in_a_graph(snapkv):
    w = Workload("graph", Hq=8, Hkv=4, D=128, L=6000, W=32, pool_kind=0, p=7, C=512, dtype="bf16",
                 clusters=(6, 6), radius=6, seed=70)
    cases = [workloads.generate(w, layer=l, device="cuda") for l in range(3)]
    q = torch.empty_like(cases[0]["q_win"])
    k = torch.empty_like(cases[0]["k"])
    v = torch.empty_like(cases[0]["v"])
    ws = torch.empty(snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W), dtype=torch.uint8, device="cuda")
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")

    def load(c):
        q.copy_(c["q_win"]); k.copy_(c["k"]); v.copy_(c["v"])

    load(cases[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture: launch plans are cached
        snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, workspace=ws)
    for rep in range(6):
        c = cases[rep % 3]
        load(c)
        out_idx.fill_(-1); out_k.zero_(); out_v.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (out_idx.cpu().numpy().copy(), out_k.clone(), out_v.clone())
        # eager call on the same inputs, own outputs, the library's own scratch
        ek = torch.zeros_like(out_k); ev = torch.zeros_like(out_v); ei = torch.zeros_like(out_idx)
        snapkv.snapkv_compress(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ek, ev, ei)
        torch.cuda.synchronize()
        assert np.array_equal(got[0], ei.cpu().numpy()), f"replay {rep}"
        assert torch.equal(got[1], ek) and torch.equal(got[2], ev), f"replay {rep}"
    assert snapkv.snapkv_sync_timeouts() == 0


def test_decode_replays_in_a_graph(snapkv):
    w = DecodeWorkload("graph_decode", B=2, Hq=8, Hkv=4, D=128, S=5000, cap=5000, seed=71)   # keys split: merge kernel too
    cases = [workloads.generate_decode(DecodeWorkload(**{**w.__dict__, "seed": 71 + i}), device="cuda") for i in range(2)]
    q = torch.empty_like(cases[0]["q"]); k = torch.empty_like(cases[0]["k_cache"]); v = torch.empty_like(cases[0]["v_cache"])
    out = torch.zeros((w.B, w.Hq, w.D), dtype=torch.float32, device="cuda")
    lse = torch.zeros((w.B, w.Hq), dtype=torch.float32, device="cuda")
    q.copy_(cases[0]["q"]); k.copy_(cases[0]["k_cache"]); v.copy_(cases[0]["v_cache"])
    snapkv.snapkv_decode_attention(q, k, v, w.S, out, lse)      # allocates the partials' buffer before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        snapkv.snapkv_decode_attention(q, k, v, w.S, out, lse)
    for rep in range(4):
        c = cases[rep % 2]
        q.copy_(c["q"]); k.copy_(c["k_cache"]); v.copy_(c["v_cache"])
        out.fill_(float("nan")); lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eo = torch.empty_like(out); el = torch.empty_like(lse)
        snapkv.snapkv_decode_attention(c["q"], c["k_cache"], c["v_cache"], w.S, eo, el)
        torch.cuda.synchronize()
        assert torch.equal(out, eo) and torch.equal(lse, el), f"replay {rep}"


def test_static_scratch_entry_replays_in_a_graph(snapkv):
    """The entry point for callers that cannot allocate is the other form to capture."""
    w = Workload("graph_static", Hq=8, Hkv=4, D=128, L=5000, W=32, pool_kind=1, p=5, C=384, dtype="bf16",
                 clusters=(6, 6), radius=6, seed=72)
    cases = [workloads.generate(w, layer=l, device="cuda") for l in range(2)]
    q = cases[0]["q_win"].clone(); k = cases[0]["k"].clone(); v = cases[0]["v"].clone()
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")
    snapkv.snapkv_compress_static(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)   # launch plans are cached
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        snapkv.snapkv_compress_static(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    for rep in range(4):
        c = cases[rep % 2]
        q.copy_(c["q_win"]); k.copy_(c["k"]); v.copy_(c["v"])
        out_idx.fill_(-1); out_k.zero_(); out_v.zero_()
        graph.replay()
        torch.cuda.synchronize()
        ek = torch.zeros_like(out_k); ev = torch.zeros_like(out_v); ei = torch.zeros_like(out_idx)
        snapkv.snapkv_compress(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ek, ev, ei)
        torch.cuda.synchronize()
        assert np.array_equal(out_idx.cpu().numpy(), ei.cpu().numpy()), f"replay {rep}"
        assert torch.equal(out_k, ek) and torch.equal(out_v, ev), f"replay {rep}"
    assert snapkv.snapkv_sync_timeouts() == 0


def test_own_scratch_entries_refuse_a_capturing_stream(snapkv):
    w = Workload("graph_refused", Hq=4, Hkv=4, D=64, L=2000, W=32, pool_kind=0, p=7, C=256, dtype="bf16",
                 clusters=(3, 3), radius=4, seed=73)
    c = workloads.generate(w, device="cuda")
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=c["k"].dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -5, dtype=torch.int32, device="cuda")
    marker = torch.zeros(8, device="cuda")
    graph = torch.cuda.CUDAGraph()
    codes = []
    with torch.cuda.graph(graph):
        marker.add_(1.0)                         # something to record
        try:
            snapkv.snapkv_compress(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
        except snapkv.SnapKVError as e:
            codes.append(e.code)
    graph.replay()
    torch.cuda.synchronize()
    assert codes == [-2]
    assert int(out_idx.min()) == -5 and int(out_idx.max()) == -5     # nothing of the call was recorded


def test_a_call_on_another_stream_prepares_the_scratch_again(snapkv):
    """The record of the state a call leaves the library's scratch in holds for the stream it was left on: a
    call on another stream is not ordered behind the kernel that left it, so the preparing launch runs."""
    w = Workload("two_streams", Hq=8, Hkv=4, D=128, L=6000, W=32, pool_kind=0, p=7, C=512, dtype="bf16",
                 clusters=(6, 6), radius=6, seed=74)
    c = workloads.generate(w, device="cuda")
    outs = [(torch.zeros((w.Hkv, w.C, w.D), dtype=c["k"].dtype, device="cuda"),
             torch.zeros((w.Hkv, w.C, w.D), dtype=c["k"].dtype, device="cuda"),
             torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")) for _ in range(3)]
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()

    def call(i, stream):
        snapkv.snapkv_profile_start(1)
        snapkv.snapkv_compress(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, *outs[i], stream=stream)
        ms, _ = snapkv.snapkv_profile_stop()      # waits for the device: the calls below never overlap
        return ms.get("prepare_scratch", 0.0) > 0.0

    call(0, a)
    assert not call(1, a)        # same stream, same shape: the last kernel left the scratch ready
    assert call(2, b)            # another stream: prepared again
    torch.cuda.synchronize()
    for i in (1, 2):
        assert torch.equal(outs[i][2], outs[0][2]) and torch.equal(outs[i][0], outs[0][0]) and torch.equal(outs[i][1], outs[0][1])


def test_long_prompt_path_replays_in_a_graph(snapkv):
    """The launches of a prompt longer than the single-read launch holds (statistics of the rest, the published
    word, the single-read kernel on the front, the votes of the rest, selection, gather) are plain kernel launches
    on the caller's workspace: captured once, replayed on other inputs, every replay equals the eager call."""
    snapkv.snapkv_set_scoring_scheme(4)
    try:
        for kw in (dict(W=32, p=7), dict(W=16, p=5)):        # the second keeps the rest's logits
            w = Workload("graph_long", Hq=4, Hkv=4, D=128, L=12000 if kw["W"] == 32 else 20000, pool_kind=0, C=384,
                         dtype="bf16", clusters=(6, 6), radius=6, seed=71, **kw)
            cases = [workloads.generate(w, layer=l, device="cuda") for l in range(2)]
            q, k, v = (torch.empty_like(cases[0][n]) for n in ("q_win", "k", "v"))
            ws = torch.empty(snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W), dtype=torch.uint8, device="cuda")
            out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
            out_v = torch.zeros_like(out_k)
            out_idx = torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")

            def load(c):
                q.copy_(c["q_win"]); k.copy_(c["k"]); v.copy_(c["v"])

            load(cases[0])
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, workspace=ws)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx, workspace=ws)
            for rep in range(4):
                c = cases[rep % 2]
                load(c)
                out_idx.fill_(-1); out_k.zero_(); out_v.zero_()
                graph.replay()
                torch.cuda.synchronize()
                ek = torch.zeros_like(out_k); ev = torch.zeros_like(out_v); ei = torch.zeros_like(out_idx)
                snapkv.snapkv_compress(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ek, ev, ei)
                torch.cuda.synchronize()
                assert torch.equal(out_idx, ei), f"replay {rep}"
                assert torch.equal(out_k, ek) and torch.equal(out_v, ev), f"replay {rep}"
        assert snapkv.snapkv_sync_timeouts() == 0
    finally:
        snapkv.snapkv_set_scoring_scheme(0)
