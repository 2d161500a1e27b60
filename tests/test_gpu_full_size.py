"""The named configurations at full size, in the launch configurations bench.py times.

The numpy oracle is evaluated on sampled KV heads (one head of the longest configuration is ~1 GFLOP of
fp64), the plain-C oracle on every head of a layer; properties that hold at any size are checked on
every head."""
import pytest
import torch

from paper_2404_14469_amd import workloads

from parity import check_against_oracle, check_self_consistency, run_gpu

pytestmark = pytest.mark.gpu


def _run(snapkv, w, layer, heads):
    print(f"[full-size] {w.name} layer {layer} L={w.L} Hq={w.Hq} Hkv={w.Hkv} oracle heads {heads}", flush=True)
    case = workloads.generate(w, layer=layer, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    res = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    check_self_consistency(q, k, v, w.C, *res)
    band = check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, heads=heads)
    print(f"[full-size] {w.name}: positions inside the +-1e-3 band around the threshold: {band}", flush=True)
    return case, res


def test_llama2_7b_16k_all_heads(snapkv):
    w = workloads.LLAMA2_7B_16K
    _run(snapkv, w, 0, list(range(w.Hkv)))


@pytest.mark.parametrize("layer", [0, 31])
def test_mistral_7b_gqa_32k(snapkv, layer):
    w = workloads.MISTRAL_7B_GQA_32K
    _run(snapkv, w, layer, list(range(w.Hkv)))


@pytest.mark.parametrize("layer,heads", [(0, [0, 13, 31]), (17, [5])])
def test_long_131k_sampled_heads_and_needle(snapkv, layer, heads):
    w = workloads.LONG_131K
    case, res = _run(snapkv, w, layer, heads)
    idx = res[3]
    for hk, pos in enumerate(case["needle_pos"]):
        lo, hi = max(0, pos - w.p // 2), min(w.n - 1, pos + w.p // 2)
        kept = set(idx[hk].tolist())
        assert set(range(lo, hi + 1)) <= kept, f"head {hk}: needle at {pos} not kept with its neighbours"
    del case, res
    torch.cuda.empty_cache()


def test_long_131k_every_head_of_a_layer_against_the_c_oracle(snapkv):
    """All 32 heads of one layer of the long-context configuration: pooled scores within 1e-3 relative of
    the plain-C fp64 oracle's, kept positions by the band rule, the kept set the exact top-k of the GPU's
    own scores, gathered rows bit-identical (the sampled heads above are the numpy oracle's second opinion)."""
    from oracle import c_oracle
    w = workloads.LONG_131K
    layer = 9
    print(f"[full-size] {w.name} layer {layer}: all {w.Hkv} heads against the plain-C oracle", flush=True)
    case = workloads.generate(w, layer=layer, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    res = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    _, _, _, kept, score = c_oracle.compress(*(workloads.to_numpy_bits(x) for x in (q, k, v)), w.W, w.pool_kind, w.p, w.C)
    assert kept == w.C and score.shape == (w.Hkv, w.n)
    band = check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, oracle_scores=score)
    print(f"[full-size] {w.name}: positions inside the +-1e-3 band around the threshold, all heads: {band}", flush=True)
    del case, res
    torch.cuda.empty_cache()


def test_layers_entry_at_full_size(snapkv):
    """Three layers of the long-context configuration through snapkv_compress_layers (stacked, so they run
    as one layer of 96 heads, on the kernels the 32-layer call of bench.py uses): bit for bit what single
    calls give, and one head against the oracle."""
    import numpy as np
    w = workloads.LONG_131K
    nl = 3
    print(f"[full-size] {w.name}: {nl} stacked layers through snapkv_compress_layers", flush=True)
    K = torch.empty((nl, w.Hkv, w.L, w.D), dtype=torch.bfloat16, device="cuda")
    V = torch.empty_like(K)
    Q = torch.empty((nl, w.Hq, w.W, w.D), dtype=torch.bfloat16, device="cuda")
    for l in range(nl):
        c = workloads.generate(w, layer=20 + l, device="cuda")
        K[l].copy_(c["k"]), V[l].copy_(c["v"]), Q[l].copy_(c["q_win"])
        del c
    ok = torch.zeros((nl, w.Hkv, w.C, w.D), dtype=torch.bfloat16, device="cuda")
    ov = torch.zeros_like(ok)
    oi = torch.full((nl, w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
    snapkv.snapkv_compress_layers(list(Q), list(K), list(V), w.pool_kind, w.p, w.C, list(ok), list(ov), list(oi))
    torch.cuda.synchronize()
    for l in range(nl):
        ref = run_gpu(snapkv, Q[l], K[l], V[l], w.pool_kind, w.p, w.C)
        assert np.array_equal(oi[l].cpu().numpy(), ref[3]), f"layer {l}: kept positions"
        assert torch.equal(ok[l], ref[1]) and torch.equal(ov[l], ref[2]), f"layer {l}: rows"
        if l == 1:
            check_against_oracle(Q[l], K[l], V[l], w.pool_kind, w.p, w.C, ref[0], ok[l], ov[l], oi[l].cpu().numpy(), w.C,
                                 heads=[17])
    assert snapkv.snapkv_sync_timeouts() == 0
    del K, V, Q, ok, ov, oi
    torch.cuda.empty_cache()


def test_window_64_pool_13_at_full_size(snapkv):
    """The wider window and pooling kernel the paper uses for one of its models (Sec. 5.4's
    Command-R setting: W = 64, p = 13), on the grouped-query and on the long configuration."""
    _run(snapkv, workloads.MISTRAL_7B_GQA_32K.with_(name="gqa_32k_w64_p13", W=64, p=13), 2, [0, 7])
    _run(snapkv, workloads.LONG_131K.with_(name="long_131k_w64_p13", W=64, p=13), 5, [11])
    torch.cuda.empty_cache()


@pytest.mark.parametrize("L,heads", [(65536, [3]), (131072, [6]), (100003, [0])])
def test_grouped_query_prompts_whose_parts_follow_one_another(snapkv, L, heads):
    """Grouped-query prompts so long that the parts of a KV head (one query head each) no longer fit
    the chip side by side: they follow one another on the same workgroups, and the single-read kernel
    still takes the prompt (two groups of two parts at 65536 tokens, one group at 131072)."""
    w = workloads.MISTRAL_7B_GQA_32K.with_(name=f"gqa_{L}", L=L, C=4096)
    snapkv.snapkv_profile_start(4)
    _run(snapkv, w, 1, heads)
    ms, calls = snapkv.snapkv_profile_stop()
    assert ms.get("score_fused", 0.0) > 0.0 and ms.get("score_stream", 0.0) == 0.0, ms
    torch.cuda.empty_cache()


def test_varlen_batch(snapkv):
    prompts = workloads.varlen_prompts()
    for i, w in enumerate(prompts):
        _run(snapkv, w, 0, [i % w.Hkv, (i + 3) % w.Hkv])


def test_varlen_batch_through_the_batch_entry(snapkv):
    """The batched-varlen configuration as bench.py times it: every prompt of the batch gets, bit for bit,
    what its own call gives (which test_varlen_batch checks against the oracle)."""
    import numpy as np
    ws = workloads.varlen_prompts()
    cases = [workloads.generate(w, device="cuda") for w in ws]
    w0 = ws[0]
    oks = [torch.zeros((w0.Hkv, w0.C, w0.D), dtype=torch.bfloat16, device="cuda") for _ in ws]
    ovs = [torch.zeros_like(t) for t in oks]
    ois = [torch.full((w0.Hkv, w0.C), -1, dtype=torch.int32, device="cuda") for _ in ws]
    kept = snapkv.snapkv_compress_varlen([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                         w0.pool_kind, w0.p, w0.C, oks, ovs, ois)
    torch.cuda.synchronize()
    for i, (w, c) in enumerate(zip(ws, cases)):
        print(f"[full-size] varlen batch prompt {i} L={w.L}", flush=True)
        ref = run_gpu(snapkv, c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C)
        assert kept[i] == ref[4] == w.C
        assert np.array_equal(ois[i].cpu().numpy(), ref[3])
        assert torch.equal(oks[i], ref[1]) and torch.equal(ovs[i], ref[2])
    assert snapkv.snapkv_sync_timeouts() == 0


def test_one_cache_per_query_head_at_full_size(snapkv):
    """The GQA configuration with one cache per query head: all properties that hold at any size on every
    query head, the oracle's per-query-head form (the step on repeated KV heads) on sampled ones."""
    w = workloads.MISTRAL_7B_GQA_32K
    case = workloads.generate(w, layer=3, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    g = w.Hq // w.Hkv
    out_k = torch.zeros((w.Hq, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hq, w.C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_per_query_head(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    k_rep, v_rep = k.repeat_interleave(g, dim=0).contiguous(), v.repeat_interleave(g, dim=0).contiguous()
    sc = torch.empty((w.Hq, w.n), dtype=torch.float32, device="cuda")
    snapkv.snapkv_pooled_scores(q, k_rep, w.pool_kind, w.p, sc)
    torch.cuda.synchronize()
    idx = out_idx.cpu().numpy()
    check_self_consistency(q, k_rep, v_rep, w.C, sc.cpu().numpy(), out_k, out_v, idx, kept)
    check_against_oracle(q, k_rep, v_rep, w.pool_kind, w.p, w.C, sc.cpu().numpy(), out_k, out_v, idx, kept,
                         heads=[0, 9, 31])


def test_paged_cache_at_full_size(snapkv):
    """The long-context configuration from 16-row pages in shuffled order: identical to the contiguous call."""
    import numpy as np
    w = workloads.LONG_131K
    case = workloads.generate(w, layer=1, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    ref = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    ps = 16
    npg = (w.L + ps - 1) // ps
    table = torch.randperm(npg, generator=torch.Generator().manual_seed(4)).to(torch.int32).cuda()
    pos = torch.arange(w.L, device="cuda")
    kp = torch.zeros((npg, ps, w.Hkv, w.D), dtype=k.dtype, device="cuda")
    vp = torch.zeros_like(kp)
    kp[table.long()[pos // ps], pos % ps] = k.permute(1, 0, 2)
    vp[table.long()[pos // ps], pos % ps] = v.permute(1, 0, 2)
    del case, k, v
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=kp.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_paged(q, kp, vp, table, w.L, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    assert kept == ref[4]
    assert np.array_equal(out_idx.cpu().numpy(), ref[3])
    assert torch.equal(out_k, ref[1]) and torch.equal(out_v, ref[2])
    assert snapkv.snapkv_sync_timeouts() == 0


def test_decode_at_full_size(snapkv):
    """The decoding workload bench.py times (batch 8, 2560 rows per head), against the oracle on two sequences."""
    import numpy as np
    from oracle import decode_oracle as dec
    w = workloads.DECODE_CAPPED_B8
    c = workloads.generate_decode(w, device="cuda")
    out = torch.empty((w.B, w.Hq, w.D), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda")
    snapkv.snapkv_decode_attention(c["q"], c["k_cache"], c["v_cache"], w.S, out, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    for b in (0, 7):
        want, want_lse = dec.decode_attention(workloads.to_numpy_bits(c["q"][b:b + 1]),
                                              workloads.to_numpy_bits(c["k_cache"][b:b + 1]),
                                              workloads.to_numpy_bits(c["v_cache"][b:b + 1]))
        vmax = float(c["v_cache"][b].float().abs().max())
        assert np.abs(out[b].cpu().numpy() - want[0]).max() <= 1e-4 * vmax
        assert np.abs(lse[b].cpu().numpy() - want_lse[0]).max() <= 1e-4


def test_two_streaming_passes_at_full_size(snapkv):
    # the path that takes over when a prompt's logits exceed the register files or the grid cannot be resident
    snapkv.snapkv_set_scoring_scheme(1)
    try:
        _run(snapkv, workloads.LLAMA2_7B_16K, 1, [0, 17])
        _run(snapkv, workloads.MISTRAL_7B_GQA_32K, 2, [3])
    finally:
        snapkv.snapkv_set_scoring_scheme(0)


def test_prompt_longer_than_the_single_read_kernel_holds(snapkv):
    # L = 200000: one head's logits no longer fit the chip's registers, so scoring takes two streaming
    # passes (row log-sum-exp, then probabilities); nothing about the result may change
    w = workloads.LONG_131K.with_(name="long_200k", L=200000, Hq=4, Hkv=4, C=2048, clusters=(16, 16), seed=77)
    case, res = _run(snapkv, w, 0, [0, 3])
    idx = res[3]
    for hk, pos in enumerate(case["needle_pos"]):
        lo, hi = max(0, pos - w.p // 2), min(w.n - 1, pos + w.p // 2)
        assert set(range(lo, hi + 1)) <= set(idx[hk].tolist())


def test_lse_entry_at_full_size(snapkv):
    # the entry point that takes the window rows' log-sum-exp, on the longest configuration and on GQA
    import numpy as np
    from oracle import snapkv_oracle as orc
    for w, layer, heads in ((workloads.LONG_131K, 2, [1, 30]), (workloads.MISTRAL_7B_GQA_32K, 5, [0, 7])):
        print(f"[full-size] lse entry {w.name} layer {layer} oracle heads {heads}", flush=True)
        case = workloads.generate(w, layer=layer, device="cuda")
        q, k, v = case["q_win"], case["k"], case["v"]
        lse = np.zeros((w.Hq, w.W), dtype=np.float32)      # rows of the sampled KV heads come from the oracle,
        g = w.Hq // w.Hkv                                   # the others stay 0 and are not compared
        for hk in heads:
            kn = workloads.to_numpy_bits(k[hk])
            for h in range(hk * g, (hk + 1) * g):
                lse[h] = orc.window_lse(workloads.to_numpy_bits(q[h]), kn).astype(np.float32)
        lt = torch.from_numpy(lse).cuda()
        sc = torch.empty((w.Hkv, w.n), dtype=torch.float32, device="cuda")
        snapkv.snapkv_pooled_scores_lse(q, k, lt, w.pool_kind, w.p, sc)
        out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
        out_v = torch.zeros_like(out_k)
        out_idx = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
        kept = snapkv.snapkv_compress_lse(q, k, v, lt, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
        torch.cuda.synchronize()
        res = (sc.cpu().numpy(), out_k, out_v, out_idx.cpu().numpy(), kept)
        check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, heads=heads)
        del case, q, k, v, out_k, out_v, sc
        torch.cuda.empty_cache()


def test_separate_pool_and_select_kernels_at_full_size(snapkv):
    # the kernels that take over when a head does not fit the cooperative pooling + selection launch
    snapkv.snapkv_set_scoring_scheme(2)
    try:
        _run(snapkv, workloads.LLAMA2_7B_16K, 1, [5, 31])
        _run(snapkv, workloads.LONG_131K, 3, [9])
    finally:
        snapkv.snapkv_set_scoring_scheme(0)


def test_many_calls_in_a_row_select_what_their_own_scores_say(snapkv):
    """The cooperative selection hands data between workgroups on different dies; a hand-over that
    a reader can overtake shows as a wrong position in a few calls out of a hundred, not in one.
    150 calls on fresh inputs (own scratch and caller's workspace alternating), each checked for
    every head against the oracle's selection from the library's own pooled scores: integer work
    on identical scores, so the comparison is exact."""
    import numpy as np
    from oracle import snapkv_oracle as orc
    w = workloads.LLAMA2_7B_16K
    ws = torch.empty(snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W), dtype=torch.uint8, device="cuda")
    kc = w.C - w.W
    for rep in range(50):
        c = workloads.generate(w, layer=rep, device="cuda")
        q, k, v = c["q_win"], c["k"], c["v"]
        sc = torch.empty((w.Hkv, w.n), dtype=torch.float32, device="cuda")
        snapkv.snapkv_pooled_scores(q, k, w.pool_kind, w.p, sc)
        got = []
        for call in range(3):
            ok = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
            ov = torch.zeros_like(ok)
            oi = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
            snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, ok, ov, oi, workspace=ws if call == 2 else None)
            got.append(oi)
        torch.cuda.synchronize()
        s0 = sc.cpu().numpy().astype(np.float64)
        want = np.stack([orc.select(s0[h], kc) for h in range(w.Hkv)])
        for call, oi in enumerate(got):
            assert np.array_equal(oi.cpu().numpy()[:, :kc], want), (rep, call)


def test_no_handoff_wait_gave_up(snapkv):
    assert snapkv.snapkv_sync_timeouts() == 0
