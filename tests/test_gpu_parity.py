"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle element by element."""
import numpy as np
import pytest
import torch

from oracle import snapkv_oracle as orc
from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload

from parity import check_against_oracle, gpu_vs_oracle, run_gpu

pytestmark = pytest.mark.gpu


def small(name, **kw):
    base = dict(Hq=4, Hkv=4, D=128, L=1000, W=32, pool_kind=0, p=7, C=160, dtype="bf16",
                clusters=(4, 4), radius=6, seed=7)
    base.update(kw)
    return Workload(name, **base)


SMALL_CASES = [
    workloads.TINY,
    small("mha_ragged"),                                     # L not a multiple of the 128-key chunk
    small("mha_one_chunk", L=100, C=48),
    small("mha_chunk_edge", L=1024 + 32, C=200),             # prefix ends exactly on a chunk edge
    small("gqa4_w32", Hq=16, Hkv=4, L=1500, C=300),
    small("gqa4_w16_avg5", Hq=16, Hkv=4, W=16, pool_kind=1, p=5, L=1337, C=200),
    small("gqa3_w16", Hq=6, Hkv=2, W=16, L=777, C=100),      # odd group: last half block is padding
    small("mha_w16", W=16, p=5, L=900, C=128),
    small("mha_w64_p13", W=64, p=13, L=1200, C=256),
    small("gqa2_w64", Hq=4, Hkv=2, W=64, p=13, L=1100, C=256),
    small("mha_w20", W=20, L=650, C=120),                    # window not a multiple of 16
    small("mha_w8_gqa8", Hq=8, Hkv=1, W=8, L=500, C=64),
    small("w1_p1", W=1, p=1, L=300, C=40),
    small("no_pool", p=1),
    small("avg_p13", pool_kind=1, p=13),
    small("d64_bf16", D=64, L=1111, C=140),
    small("f32_d128", dtype="f32", L=800, C=130),
    small("f32_d64_gqa", dtype="f32", D=64, Hq=8, Hkv=2, W=16, pool_kind=1, p=5, L=600, C=90),
    small("c_equals_w", C=32),                               # nothing selected, window only
    small("c_is_l_minus_1", L=200, C=199),                   # exactly one position dropped
    small("tiny_prefix", L=40, W=32, C=36),                  # n = 8 < one tile
    small("l_is_w_plus_1", L=33, W=32, C=32),
    small("needle", L=4096, C=256, needle=True, clusters=(8, 8)),
    small("mha_w160", W=160, L=1300, C=320, p=5),            # more window rows than a wave tracks
    small("f16_d128", dtype="f16", L=1234, C=150),
    small("f16_d64_gqa", dtype="f16", D=64, Hq=8, Hkv=2, W=16, pool_kind=1, p=5, L=700, C=100),
    small("f16_w160", dtype="f16", W=160, L=900, C=200),
]


@pytest.fixture(params=[0, 1, 2], ids=["single_read", "two_streaming_passes", "separate_pool_select"])
def scheme(request, snapkv):
    """The default path (single-read scoring, pooling + selection in one launch), scoring in two
    streaming passes with nothing handed between workgroups, and the separate pooling and
    selection kernels."""
    snapkv.snapkv_set_scoring_scheme(request.param)
    yield request.param
    snapkv.snapkv_set_scoring_scheme(0)
    assert snapkv.snapkv_sync_timeouts() == 0


@pytest.mark.parametrize("w", SMALL_CASES, ids=lambda w: w.name)
def test_small_cases_all_heads(snapkv, scheme, w):
    case, res, band = gpu_vs_oracle(snapkv, w)
    if w.needle:
        idx = res[3]
        for hk, pos in enumerate(case["needle_pos"]):
            lo, hi = max(0, pos - w.p // 2), min(w.n - 1, pos + w.p // 2)
            assert set(range(lo, hi + 1)) <= set(idx[hk].tolist())


@pytest.mark.parametrize("L,C", [(64, 64), (50, 128), (32, 32)])
def test_bypass_identity(snapkv, L, C):
    w = small("bypass", L=L, C=C)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    out_k = torch.full((w.Hkv, C, w.D), 7.0, dtype=k.dtype, device="cuda")
    out_v = torch.full((w.Hkv, C, w.D), 7.0, dtype=k.dtype, device="cuda")
    out_idx = torch.full((w.Hkv, C), -5, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress(q, k, v, 0, 7, C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    assert kept == L
    assert torch.equal(out_k[:, :L], k) and torch.equal(out_v[:, :L], v)
    assert torch.equal(out_idx[:, :L].cpu(), torch.arange(L, dtype=torch.int32).expand(w.Hkv, L))
    # rows [L, C) are documented as not written
    assert bool((out_idx[:, L:] == -5).all()) and bool((out_k[:, L:] == 7.0).all())


def test_zero_queries_flat_field_tie_rule(snapkv, scheme):
    # all-zero queries: every prefix vote equals H_L - H_n, so max pooling gives a flat field
    # and the tie rule alone decides: positions 0..k-1 (closed form, not an oracle call)
    w = small("flat", L=2000, C=500)
    case = workloads.generate(w, device="cuda")
    q = torch.zeros_like(case["q_win"])
    scores, out_k, out_v, idx, kept = run_gpu(snapkv, q, case["k"], case["v"], 0, 7, w.C)
    h = sum(1.0 / t for t in range(w.n + 1, w.L + 1))
    assert np.allclose(scores, h, rtol=1e-5)
    want = np.concatenate([np.arange(w.C - w.W), np.arange(w.n, w.L)])
    for hk in range(w.Hkv):
        assert np.array_equal(idx[hk], want)


def test_zero_queries_avgpool_skips_edges(snapkv):
    w = small("flat_avg", L=2000, C=500, pool_kind=1, p=5)
    case = workloads.generate(w, device="cuda")
    q = torch.zeros_like(case["q_win"])
    scores, _, _, idx, _ = run_gpu(snapkv, q, case["k"], case["v"], 1, 5, w.C)
    h = sum(1.0 / t for t in range(w.n + 1, w.L + 1))
    assert np.allclose(scores[:, 2:w.n - 2], h, rtol=1e-5)
    assert np.allclose(scores[:, [0, w.n - 1]], h * 3 / 5, rtol=1e-5)
    assert np.allclose(scores[:, [1, w.n - 2]], h * 4 / 5, rtol=1e-5)
    assert idx[:, :w.C - w.W].min() >= 2 and idx[:, :w.C - w.W].max() <= w.n - 3


def test_shift_invariance_large_offset(snapkv, scheme):
    # one vector added to every key shifts whole rows of logits by a constant (here ~100 nats,
    # enough to overflow a softmax without max subtraction); selection must not change and the
    # scores must still match the oracle evaluated on the shifted bytes
    w = small("shift", L=1500, C=200, dtype="f32", D=64)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    qm = q.mean(dim=(0, 1))
    k2 = (k + 250.0 * qm / qm.norm()).contiguous()
    shift = (q.reshape(-1, w.D) @ (250.0 * qm / qm.norm())) / 8.0
    assert float(shift.max()) > 89.0
    res = run_gpu(snapkv, q, k2, v, 0, 7, w.C)
    assert np.all(np.isfinite(res[0]))
    check_against_oracle(q, k2, v, 0, 7, w.C, *res)


def test_deterministic_bitwise(snapkv, scheme):
    w = small("det", Hq=8, Hkv=2, L=3000, C=400)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    a = run_gpu(snapkv, q, k, v, 0, 7, w.C)
    b = run_gpu(snapkv, q, k, v, 0, 7, w.C)
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32))
    assert np.array_equal(a[3], b[3])
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def _compress_only(snapkv, case, w):
    q, k, v = case["q_win"], case["k"], case["v"]
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    assert kept == w.C
    return out_idx.cpu().numpy(), out_k, out_v


def test_back_to_back_calls_reuse_the_scratch_state(snapkv):
    """Consecutive calls of one shape skip the preparing launch (the previous call's last kernel
    left the scratch ready); other shapes, other entry points and other schemes in between must
    not leave anything stale behind."""
    wa = small("b2b_a", Hq=8, Hkv=4, L=5000, C=600)
    wb = small("b2b_b", Hq=4, Hkv=4, L=3100, C=200, pool_kind=1, p=5)
    ca = workloads.generate(wa, device="cuda")
    ca2 = workloads.generate(wa.with_(seed=wa.seed + 7), device="cuda")
    cb = workloads.generate(wb, device="cuda")
    ref_a = run_gpu(snapkv, ca["q_win"], ca["k"], ca["v"], wa.pool_kind, wa.p, wa.C)
    check_against_oracle(ca["q_win"], ca["k"], ca["v"], wa.pool_kind, wa.p, wa.C, *ref_a)
    ref_a2 = run_gpu(snapkv, ca2["q_win"], ca2["k"], ca2["v"], wa.pool_kind, wa.p, wa.C)
    ref_b = run_gpu(snapkv, cb["q_win"], cb["k"], cb["v"], wb.pool_kind, wb.p, wb.C)

    def same(got, ref):
        assert np.array_equal(got[0], ref[3])
        assert torch.equal(got[1], ref[1]) and torch.equal(got[2], ref[2])

    for _ in range(3):                                  # same shape, back to back
        same(_compress_only(snapkv, ca, wa), ref_a)
        same(_compress_only(snapkv, ca2, wa), ref_a2)
    same(_compress_only(snapkv, cb, wb), ref_b)         # another shape in between
    same(_compress_only(snapkv, ca, wa), ref_a)
    same(_compress_only(snapkv, ca, wa), ref_a)
    sc = torch.empty((wa.Hkv, wa.n), dtype=torch.float32, device="cuda")
    snapkv.snapkv_pooled_scores(ca["q_win"], ca["k"], wa.pool_kind, wa.p, sc)   # another entry point
    same(_compress_only(snapkv, ca2, wa), ref_a2)
    same(_compress_only(snapkv, ca2, wa), ref_a2)
    for sch in (1, 2, 0):                               # other schemes in between
        snapkv.snapkv_set_scoring_scheme(sch)
        try:
            got = _compress_only(snapkv, ca, wa)
        finally:
            snapkv.snapkv_set_scoring_scheme(0)
        assert np.array_equal(got[0], ref_a[3]) or sch == 1   # two-pass scores may differ in the last bit
        same(_compress_only(snapkv, ca, wa), ref_a)
    assert snapkv.snapkv_sync_timeouts() == 0


def test_prompts_of_differing_length_back_to_back(snapkv):
    """A batch of prompts of one model but different lengths, compressed one after the other in
    any order: the ready state of the scratch carries over from longer to shorter prompts and
    back, and every call still matches the oracle."""
    lengths = [9000, 2300, 30000, 700, 30000, 5100, 9000]
    cases = {}
    for L in sorted(set(lengths)):
        w = small(f"mix_{L}", Hq=8, Hkv=2, L=L, C=min(400, L // 2), seed=L)
        cases[L] = (w, workloads.generate(w, device="cuda"))
    refs = {}
    for L, (w, c) in cases.items():
        refs[L] = run_gpu(snapkv, c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C)
        check_against_oracle(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, *refs[L])
    for rounds in range(2):
        for L in lengths:
            w, c = cases[L]
            got = _compress_only(snapkv, c, w)
            assert np.array_equal(got[0], refs[L][3]), L
            assert torch.equal(got[1], refs[L][1]) and torch.equal(got[2], refs[L][2]), L
    assert snapkv.snapkv_sync_timeouts() == 0


def _per_query_head(snapkv, w, case):
    q, k, v = case["q_win"], case["k"], case["v"]
    out_k = torch.zeros((w.Hq, w.C, w.D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hq, w.C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_per_query_head(q, k, v, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    return out_k, out_v, out_idx.cpu().numpy(), kept


PER_HEAD_CASES = [
    (small("pqh_gqa4_w32", Hq=16, Hkv=4, L=2200, C=300), True),      # same launch shape as the repeated-head run
    (small("pqh_gqa2_w16", Hq=8, Hkv=4, L=1500, W=16, C=200, pool_kind=1, p=5), False),
    (small("pqh_gqa8_d64", Hq=16, Hkv=2, D=64, L=3000, W=32, C=256, p=13), False),
    (small("pqh_mha", Hq=4, Hkv=4, L=1300, C=160), True),
    (small("pqh_f16", Hq=8, Hkv=2, L=1800, C=256, dtype="f16"), False),
    (small("pqh_bypass", Hq=8, Hkv=2, L=120, C=160), True),
    (small("pqh_two_pass_select", Hq=8, Hkv=2, L=40000, C=1024), False),
]


@pytest.mark.parametrize("w,exact", PER_HEAD_CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_one_cache_per_query_head(snapkv, scheme, w, exact):
    """snapkv_compress_per_query_head against the oracle's per-query-head form, which is the
    equal-head-count step on KV heads repeated g times: the checker gets the repeated tensors."""
    case = workloads.generate(w, device="cuda")
    out_k, out_v, out_idx, kept = _per_query_head(snapkv, w, case)
    g = w.Hq // w.Hkv
    k_rep = case["k"].repeat_interleave(g, dim=0).contiguous()
    v_rep = case["v"].repeat_interleave(g, dim=0).contiguous()
    scores = None
    if w.L > w.C:
        sc = torch.empty((w.Hq, w.n), dtype=torch.float32, device="cuda")
        snapkv.snapkv_pooled_scores(case["q_win"], k_rep, w.pool_kind, w.p, sc)
        scores = sc.cpu().numpy()
    check_against_oracle(case["q_win"], k_rep, v_rep, w.pool_kind, w.p, w.C, scores, out_k, out_v, out_idx, kept,
                         own_topk_exact=exact and scheme != 1)
    assert snapkv.snapkv_sync_timeouts() == 0


def test_per_query_head_equals_grouped_call_without_groups(snapkv):
    w = small("pqh_eq", Hq=4, Hkv=4, L=2100, C=256)
    case = workloads.generate(w, device="cuda")
    a = _per_query_head(snapkv, w, case)
    b = _compress_only(snapkv, case, w)
    assert np.array_equal(a[2], b[0]) and torch.equal(a[0], b[1]) and torch.equal(a[1], b[2])


def _paged(case, w, page_size, seed):
    """Scatters the contiguous K/V of a case into pages [num_pages, page_size, Hkv, D] behind a random table
    (torch indexing only: input preparation); unused pages and the tail of the last page hold large values."""
    k, v = case["k"], case["v"]
    nlog = (w.L + page_size - 1) // page_size
    num_pages = nlog + 3
    g = torch.Generator().manual_seed(seed)
    table = torch.randperm(num_pages, generator=g)[:nlog].to(torch.int32)
    kp = torch.full((num_pages, page_size, w.Hkv, w.D), 3.0e4, dtype=k.dtype, device="cuda")
    vp = torch.full_like(kp, -3.0e4)
    pos = torch.arange(w.L)
    phys_page = table.long()[pos // page_size].cuda()
    in_page = (pos % page_size).cuda()
    kp[phys_page, in_page] = k.permute(1, 0, 2)
    vp[phys_page, in_page] = v.permute(1, 0, 2)
    return kp, vp, table.cuda()


PAGED_CASES = [
    (small("paged_16", L=1500, C=200), 16),
    (small("paged_64_gqa", Hq=16, Hkv=4, L=3000, C=300), 64),
    (small("paged_48_ragged", L=1111, C=140), 48),                   # not a power of two, L not a multiple
    (small("paged_1", L=300, C=64), 1),                              # every row its own page
    (small("paged_256_d64_f16", D=64, dtype="f16", L=2500, C=256), 256),
    (small("paged_w160", W=160, L=1300, C=320, p=5), 32),            # the wide-window kernels
    (small("paged_bypass", L=100, C=128), 16),
    (small("paged_one_page", L=200, C=64), 512),                     # the whole prompt inside one page
]


@pytest.mark.parametrize("w,page_size", PAGED_CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_paged_cache_matches_contiguous_and_oracle(snapkv, scheme, w, page_size):
    from oracle import snapkv_oracle as orc_
    case = workloads.generate(w, device="cuda")
    kp, vp, table = _paged(case, w, page_size, seed=w.L)
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=kp.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_paged(case["q_win"], kp, vp, table, w.L, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    ref = run_gpu(snapkv, case["q_win"], case["k"], case["v"], w.pool_kind, w.p, w.C)
    rows = min(w.C, w.L)
    assert kept == ref[4]
    assert np.array_equal(out_idx.cpu().numpy()[:, :rows], ref[3][:, :rows])
    assert torch.equal(out_k[:, :rows], ref[1][:, :rows]) and torch.equal(out_v[:, :rows], ref[2][:, :rows])
    # against the oracle on its own logical view of the pages
    kl = orc_.rows_from_pages(workloads.to_numpy_bits(kp), table.cpu().numpy(), w.L)
    vl = orc_.rows_from_pages(workloads.to_numpy_bits(vp), table.cpu().numpy(), w.L)
    assert np.array_equal(kl, workloads.to_numpy_bits(case["k"])) and np.array_equal(vl, workloads.to_numpy_bits(case["v"]))
    check_against_oracle(case["q_win"], case["k"], case["v"], w.pool_kind, w.p, w.C, ref[0], out_k, out_v,
                         out_idx.cpu().numpy(), kept)


def test_paged_rejects_bad_arguments(snapkv):
    w = small("paged_bad", L=500, C=64)
    case = workloads.generate(w, device="cuda")
    kp, vp, table = _paged(case, w, 16, seed=1)
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=kp.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")
    lib = snapkv.load()
    args = lambda npages, ps: (0, case["q_win"].data_ptr(), kp.data_ptr(), vp.data_ptr(), table.data_ptr(), npages, ps,
                               w.L, w.Hq, w.Hkv, w.D, w.W, 0, 7, w.C, out_k.data_ptr(), out_v.data_ptr(),
                               out_idx.data_ptr(), None)
    assert lib.snapkv_compress_paged(*args(10, 16)) == -1      # the prompt needs 32 pages
    assert lib.snapkv_compress_paged(*args(40, 0)) == -1


def test_explicit_workspace_matches(snapkv):
    w = small("ws", Hq=8, Hkv=4, L=2500, C=300)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    ref = run_gpu(snapkv, q, k, v, 0, 7, w.C)
    need = snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out_k = torch.zeros_like(ref[1])
    out_v = torch.zeros_like(ref[2])
    out_idx = torch.zeros((w.Hkv, w.C), dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress(q, k, v, 0, 7, w.C, out_k, out_v, out_idx, workspace=ws)
    torch.cuda.synchronize()
    assert kept == w.C
    assert np.array_equal(out_idx.cpu().numpy(), ref[3])
    assert torch.equal(out_k, ref[1]) and torch.equal(out_v, ref[2])
    with pytest.raises(snapkv.SnapKVError) as e:
        snapkv.snapkv_compress(q, k, v, 0, 7, w.C, out_k, out_v, out_idx, workspace=ws[:need - 256])
    assert e.value.code == -4


# ----------------------------------------------------------------------------- handed-in log-sum-exp
def _oracle_lse(q, k):
    """[Hq, W] float32 from the fp64 oracle (never from the GPU)."""
    qn, kn = workloads.to_numpy_bits(q), workloads.to_numpy_bits(k)
    g = qn.shape[0] // kn.shape[0]
    return np.stack([orc.window_lse(qn[h], kn[h // g]) for h in range(qn.shape[0])]).astype(np.float32)


def _run_lse(snapkv, q, k, v, lse, pool_kind, p, C):
    Hkv, L, D = k.shape
    W = q.shape[1]
    sc = torch.full((Hkv, L - W), float("nan"), dtype=torch.float32, device="cuda")
    snapkv.snapkv_pooled_scores_lse(q, k, lse, pool_kind, p, sc)
    out_k = torch.zeros((Hkv, C, D), dtype=k.dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((Hkv, C), -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_lse(q, k, v, lse, pool_kind, p, C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    return sc.cpu().numpy(), out_k, out_v, out_idx.cpu().numpy(), kept


LSE_CASES = [w for w in SMALL_CASES if w.L > w.C and w.L > w.W and w.W <= 128]


@pytest.mark.parametrize("w", LSE_CASES, ids=lambda w: w.name)
def test_lse_entry_small_cases(snapkv, w):
    # with the rows' own log-sum-exp the result must meet the same bar against the same oracle
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    lse = torch.from_numpy(_oracle_lse(q, k)).cuda()
    res = _run_lse(snapkv, q, k, v, lse, w.pool_kind, w.p, w.C)
    check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res)


def test_lse_offset_scales_rows_on_the_gpu(snapkv):
    # the oracle's row-scaling law: lse + d_i scales row i by exp(-d_i); compared with the oracle
    # given the same (wrong on purpose) lse
    w = small("lse_off", Hq=4, Hkv=2, L=1500, C=200, W=16, p=5)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    lse = _oracle_lse(q, k)
    rng = np.random.default_rng(5)
    lse_off = (lse + rng.uniform(-1.0, 2.0, size=lse.shape)).astype(np.float32)
    sc = torch.empty((w.Hkv, w.n), dtype=torch.float32, device="cuda")
    snapkv.snapkv_pooled_scores_lse(q, k, torch.from_numpy(lse_off).cuda(), w.pool_kind, w.p, sc)
    torch.cuda.synchronize()
    want = orc.pooled_scores(workloads.to_numpy_bits(q), workloads.to_numpy_bits(k), w.W, w.pool_kind, w.p,
                             lse=lse_off.astype(np.float64))
    assert np.allclose(sc.cpu().numpy(), want, rtol=1e-3, atol=1e-30)


# ----------------------------------------------------------------------------- strided K / V
@pytest.mark.parametrize("w", [small("tm_mha", L=2100, C=300), small("tm_gqa_f32", dtype="f32", D=64, Hq=8, Hkv=2,
                                                                       W=16, pool_kind=1, p=5, L=900, C=120),
                               small("tm_bypass", L=100, C=128)], ids=lambda w: w.name)
def test_strided_layouts_match_contiguous(snapkv, w):
    # the same logical [Hkv, L, D] tensors stored token-major and with padded rows must give what the
    # contiguous call gives, bit for bit (which is itself checked against the oracle)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    ref = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    if w.L > w.C:
        check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *ref)
    k_tm = k.permute(1, 0, 2).contiguous().permute(1, 0, 2)            # storage [L, Hkv, D]
    v_pad = torch.zeros((w.Hkv, w.L, w.D + 8), dtype=v.dtype, device="cuda")
    v_pad[..., : w.D] = v
    v_view = v_pad[..., : w.D]                                          # row stride D + 8
    assert not k_tm.is_contiguous() and not v_view.is_contiguous()
    out_k = torch.zeros_like(ref[1])
    out_v = torch.zeros_like(ref[2])
    out_idx = torch.full(ref[3].shape, -1, dtype=torch.int32, device="cuda")
    kept = snapkv.snapkv_compress_strided(q, k_tm, v_view, w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    assert kept == ref[4]
    assert np.array_equal(out_idx.cpu().numpy()[:, :kept], ref[3][:, :kept])
    assert torch.equal(out_k[:, :kept], ref[1][:, :kept]) and torch.equal(out_v[:, :kept], ref[2][:, :kept])


# ----------------------------------------------------------------------------- selector alone
def _select_case(snapkv, scores_np, kcount):
    s = torch.from_numpy(scores_np).cuda()
    out = torch.full((s.shape[0], kcount), -1, dtype=torch.int32, device="cuda")
    snapkv.snapkv_select_topk(s, kcount, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for h in range(s.shape[0]):
        want = orc.select(scores_np[h].astype(np.float64), kcount)
        assert np.array_equal(got[h], want), f"row {h}"


@pytest.mark.parametrize("n,kcount", [(1, 1), (63, 10), (64, 64), (1000, 1), (1000, 999),
                                      (5000, 777), (131040, 4064), (20001, 20001)])
def test_select_random(snapkv, n, kcount):
    rng = np.random.default_rng(n + kcount)
    _select_case(snapkv, rng.random((3, n)).astype(np.float32), kcount)


def test_select_heavy_ties(snapkv):
    rng = np.random.default_rng(5)
    n = 30000
    few = rng.integers(0, 7, size=(4, n)).astype(np.float32) * 0.125     # 7 distinct values
    _select_case(snapkv, few, 5000)
    _select_case(snapkv, np.full((2, n), 0.5, dtype=np.float32), 1234)   # all equal
    _select_case(snapkv, np.zeros((2, n), dtype=np.float32), 17)          # all +0
    runs = np.repeat(rng.random((2, n // 6)).astype(np.float32), 6, axis=1)  # pooled-style runs
    _select_case(snapkv, runs, 4001)


def test_select_wide_dynamic_range(snapkv):
    rng = np.random.default_rng(6)
    n = 40000
    x = np.exp(rng.uniform(-80, 3, size=(3, n))).astype(np.float32)       # spans many exponents
    x[:, ::97] = 0.0
    x[0, 5] = np.float32(1e-45)                                           # a denormal
    _select_case(snapkv, x, 3000)
    _select_case(snapkv, x, n - 5)


def _random_shapes(seed, count, windows=(1, 2, 7, 8, 15, 16, 17, 31, 32, 33, 48, 64)):
    import random
    rng = random.Random(seed)
    out = []
    for it in range(count):
        g = rng.choice([1, 1, 2, 4, 8])
        Hkv = rng.choice([1, 2, 3, 4, 8])
        W = rng.choice(list(windows))
        n = rng.choice([1, 2, 5, 17, 63, 64, 65, 255, 300, 511, 512, 513, 1000, 2047, 2048, 2049, 3000, 4100, 5000,
                        7001, 9000])
        C = W + rng.choice([0, 1, 2, max(1, n // 7), max(1, n // 2), max(0, n - 1), n, n + 5])
        out.append(Workload(f"random{seed}_{it}", Hq=Hkv * g, Hkv=Hkv, D=rng.choice([64, 128]), L=W + n, W=W,
                            pool_kind=rng.choice([0, 1]), p=rng.choice([1, 3, 5, 7, 13, 21, 129]), C=C,
                            dtype=rng.choice(["bf16", "bf16", "f16", "f32"]), clusters=(1, 4),
                            radius=rng.choice([1, 4, 9]), seed=1000 + it))
    return out


@pytest.mark.parametrize("w", _random_shapes(7, 64), ids=lambda w: w.name)
def test_random_shapes(snapkv, w):
    """Shapes nobody picked by hand: head counts, windows, prefix lengths, pooling widths, capacities and
    storage types drawn from lists that straddle the kernels' tile, chunk and wave sizes (capacity 0, 1,
    all but one, all, and more than all of the prefix included), each against the oracle."""
    gpu_vs_oracle(snapkv, w)


@pytest.mark.parametrize("w", _random_shapes(21, 48, windows=(64, 64, 96, 128)), ids=lambda w: w.name)
def test_random_shapes_with_long_windows(snapkv, w):
    """Windows of two, three and four 32-row blocks: the single-read kernel scores them block by block
    (one vote row per block, summed before pooling); head counts, lengths, pooling and capacities as above."""
    gpu_vs_oracle(snapkv, w)


def test_window_lengths_the_kernels_do_not_take_are_refused(snapkv):
    """More than 128 window rows go through the kernels in whole 32-row blocks; other lengths are refused
    before anything is enqueued (outputs untouched)."""
    w = small("w130", W=130, L=900, C=300)
    case = workloads.generate(w, device="cuda")
    out_k = torch.zeros((w.Hkv, w.C, w.D), dtype=case["k"].dtype, device="cuda")
    out_v = torch.zeros_like(out_k)
    out_idx = torch.full((w.Hkv, w.C), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_compress(case["q_win"], case["k"], case["v"], w.pool_kind, w.p, w.C, out_k, out_v, out_idx)
    torch.cuda.synchronize()
    assert int(out_idx.min()) == -7 and int(out_idx.max()) == -7
    sc = torch.zeros((w.Hkv, w.n), dtype=torch.float32, device="cuda")
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_pooled_scores(case["q_win"], case["k"], w.pool_kind, w.p, sc)


def test_random_sweep_across_schemes(snapkv):
    """400 more drawn shapes in one test, each under a drawn kernel scheme (single-read or two streaming passes,
    cooperative or chunked selection, the plans counting 16 resident workgroups or all), each against the oracle;
    every third one also as a list of separately allocated layers, which must equal the single call bit for bit."""
    import random
    rng = random.Random(20240414)
    for it in range(400):
        scheme = rng.choice([0, 0, 0, 1, 2, 4, 4, 5, 6])
        g, Hkv = rng.choice([1, 1, 2, 4, 8]), rng.choice([1, 2, 3, 4, 8])
        W = rng.choice([1, 2, 7, 8, 15, 16, 17, 31, 32, 33, 48, 64, 96, 128, 160])
        n = rng.choice([1, 2, 5, 17, 63, 64, 65, 255, 300, 511, 512, 513, 1000, 2047, 2048, 2049, 3000, 4100, 5000, 7001, 9000,
                        12289, 16400, 20000])
        C = W + rng.choice([0, 1, 2, max(1, n // 7), max(1, n // 2), max(0, n - 1), n, n + 5])
        w = Workload(f"sweep{it}", Hq=Hkv * g, Hkv=Hkv, D=rng.choice([64, 128]), L=W + n, W=W, pool_kind=rng.choice([0, 1]),
                     p=rng.choice([1, 3, 5, 7, 13, 21, 129]), C=C, dtype=rng.choice(["bf16", "bf16", "f16", "f32"]),
                     clusters=(1, 4), radius=rng.choice([1, 4, 9]), seed=rng.randrange(1 << 30))
        what = f"case {it}: scheme {scheme}, {w}"
        snapkv.snapkv_set_scoring_scheme(scheme)
        try:
            case = workloads.generate(w, device="cuda")
            q, k, v = case["q_win"], case["k"], case["v"]
            res = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
            try:
                check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, own_topk_exact=(scheme & 1) == 0)
            except AssertionError as e:
                raise AssertionError(f"{what}: {e}") from e
            if w.L > w.C and it % 3 == 0:
                qs, ks, vs = ([t.clone() for _ in range(2)] for t in (q, k, v))
                oks, ovs = [torch.zeros_like(res[1]) for _ in range(2)], [torch.zeros_like(res[2]) for _ in range(2)]
                ois = [torch.full(res[3].shape, -1, dtype=torch.int32, device="cuda") for _ in range(2)]
                snapkv.snapkv_compress_layers(qs, ks, vs, w.pool_kind, w.p, w.C, oks, ovs, ois)
                torch.cuda.synchronize()
                for l in range(2):
                    assert np.array_equal(ois[l].cpu().numpy(), res[3]), what
                    assert torch.equal(oks[l], res[1]) and torch.equal(ovs[l], res[2]), what
        finally:
            snapkv.snapkv_set_scoring_scheme(0)
    assert snapkv.snapkv_sync_timeouts() == 0
