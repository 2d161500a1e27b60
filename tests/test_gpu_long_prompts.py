"""Prompts of which one head's window logits do not fit the chip's registers: the single-read kernel scores
the keys that fit, two streaming passes the rest, and the two parts share one softmax (Eq. 1).  With scheme
bit 2 the plans count 16 resident workgroups, so prompts of a few thousand tokens take that path and the
oracle checks every head; the full-size cases check sampled heads."""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload
from parity import check_against_oracle, gpu_vs_oracle, run_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture()
def few_slots(snapkv):
    snapkv.snapkv_set_scoring_scheme(4)
    try:
        yield snapkv
    finally:
        snapkv.snapkv_set_scoring_scheme(0)


BASE = dict(L=20000, Hq=8, Hkv=8, D=128, W=32, pool_kind=0, p=7, C=512, dtype="bf16", clusters=(6, 6), radius=6,
            layers=1, seed=5200)

# front part: 16 workgroups of 512 keys (two row units), 1024 (one) or fewer (more row units per unit)
SHAPES = {
    "mha_w32": dict(),
    "mha_w32_rest_shorter_than_a_tile": dict(L=8192 + 32 + 5),
    "mha_w32_rest_is_window_plus_one": dict(L=8192 + 33),
    "mha_w16_avg": dict(W=16, p=5, pool_kind=1, L=30011, C=300),
    "gqa4_w32": dict(Hq=16, Hkv=4, L=17000),
    "gqa4_w16": dict(Hq=16, Hkv=4, W=16, L=9000, C=200),
    "gqa2_w8": dict(Hq=8, Hkv=4, W=8, L=12345, C=128),
    "w64_p13": dict(W=64, p=13, L=9999, C=600),
    "f16_d64": dict(dtype="f16", D=64, L=13000),
    "f32": dict(dtype="f32", Hq=4, Hkv=4, L=11000, C=256),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_front_and_rest_share_one_softmax(few_slots, name):
    kw = dict(BASE)
    kw.update(SHAPES[name])
    w = Workload("long_" + name, **kw)
    gpu_vs_oracle(few_slots, w)
    assert few_slots.snapkv_sync_timeouts() == 0


def test_same_selection_as_two_streaming_passes(few_slots):
    """The path changes how the keys are read, not what is kept: positions equal the two-pass path's wherever
    that one's scores are not within rounding of the threshold (checked through the oracle band on both)."""
    w = Workload("long_cmp", **dict(BASE, L=25000, Hq=4, Hkv=4))
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    a = run_gpu(few_slots, q, k, v, w.pool_kind, w.p, w.C)
    few_slots.snapkv_set_scoring_scheme(1)
    b = run_gpu(few_slots, q, k, v, w.pool_kind, w.p, w.C)
    few_slots.snapkv_set_scoring_scheme(4)
    assert np.abs(a[0] - b[0]).max() <= 2e-6 * np.abs(b[0]).max()
    for hk in range(w.Hkv):
        assert len(set(a[3][hk].tolist()) ^ set(b[3][hk].tolist())) <= 4
    check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *a)


def test_layers_entry_and_repeated_calls(few_slots):
    """Stacked layers pass as one layer of more heads through the same launches; calls in a row reuse the
    hand-off words the gather re-arms."""
    w = Workload("long_layers", **dict(BASE, L=12000, Hq=4, Hkv=4, C=256))
    cases = [workloads.generate(w, layer=l, device="cuda") for l in range(3)]
    q, k, v = (torch.stack([c[n] for c in cases]).contiguous() for n in ("q_win", "k", "v"))
    for _ in range(3):
        ok = torch.zeros((3, w.Hkv, w.C, w.D), dtype=k.dtype, device="cuda")
        ov = torch.zeros_like(ok)
        oi = torch.full((3, w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
        few_slots.snapkv_compress_layers(list(q), list(k), list(v), w.pool_kind, w.p, w.C, list(ok), list(ov), list(oi))
        torch.cuda.synchronize()
        for l in range(3):
            ref = run_gpu(few_slots, q[l], k[l], v[l], w.pool_kind, w.p, w.C)
            assert np.array_equal(oi[l].cpu().numpy(), ref[3])
            assert torch.equal(ok[l], ref[1]) and torch.equal(ov[l], ref[2])
    check_against_oracle(q[2], k[2], v[2], w.pool_kind, w.p, w.C, *ref)
    assert few_slots.snapkv_sync_timeouts() == 0


@pytest.mark.parametrize("L,W,p,C,heads", [(262144, 32, 7, 4096, [0, 5]), (380000, 16, 5, 1024, [1, 6])])
def test_full_size_long_prompts(snapkv, L, W, p, C, heads):
    """262144 tokens at the long-context setting's window, and the 380K-token setting of Sec. 5.1.1
    (C = 1024, max pooling over 5, W = 16), eight heads resident, sampled heads against the oracle."""
    w = workloads.LONG_131K.with_(name=f"long_{L}", L=L, W=W, p=p, C=C, Hq=8, Hkv=8, clusters=(16, 16), seed=78)
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    res = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *res, heads=heads)
    idx = res[3]
    for hk, pos in enumerate(case["needle_pos"]):
        lo, hi = max(0, pos - w.p // 2), min(w.n - 1, pos + w.p // 2)
        assert set(range(lo, hi + 1)) <= set(idx[hk].tolist())
    assert snapkv.snapkv_sync_timeouts() == 0


def test_other_entries_on_prompts_beyond_the_single_read_length(few_slots):
    """Token-major K (the rest starts at an address offset, whatever the row stride), paged K (the rest starts at
    a logical row of the page table) and one cache per query head: each equals the plain call."""
    from test_gpu_parity import _paged
    snapkv = few_slots
    w = Workload("long_entries", **dict(BASE, L=12000, Hq=8, Hkv=4, C=384))
    case = workloads.generate(w, device="cuda")
    q, k, v = case["q_win"], case["k"], case["v"]
    ref = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
    check_against_oracle(q, k, v, w.pool_kind, w.p, w.C, *ref)

    def fresh():
        return (torch.zeros_like(ref[1]), torch.zeros_like(ref[2]),
                torch.full(ref[3].shape, -1, dtype=torch.int32, device="cuda"))

    k_tm = k.permute(1, 0, 2).contiguous().permute(1, 0, 2)            # storage [L, Hkv, D]
    v_tm = v.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    ok, ov, oi = fresh()
    assert snapkv.snapkv_compress_strided(q, k_tm, v_tm, w.pool_kind, w.p, w.C, ok, ov, oi) == w.C
    torch.cuda.synchronize()
    assert np.array_equal(oi.cpu().numpy(), ref[3]) and torch.equal(ok, ref[1]) and torch.equal(ov, ref[2])

    kp, vp, table = _paged(case, w, 16, seed=5)
    ok, ov, oi = fresh()
    assert snapkv.snapkv_compress_paged(q, kp, vp, table, w.L, w.pool_kind, w.p, w.C, ok, ov, oi) == w.C
    torch.cuda.synchronize()
    assert np.array_equal(oi.cpu().numpy(), ref[3]) and torch.equal(ok, ref[1]) and torch.equal(ov, ref[2])

    okq = torch.zeros((w.Hq, w.C, w.D), dtype=k.dtype, device="cuda")
    ovq = torch.zeros_like(okq)
    oiq = torch.full((w.Hq, w.C), -1, dtype=torch.int32, device="cuda")
    assert snapkv.snapkv_compress_per_query_head(q, k, v, w.pool_kind, w.p, w.C, okq, ovq, oiq) == w.C
    torch.cuda.synchronize()
    g = w.Hq // w.Hkv
    for h in range(w.Hq):          # each query head alone is a prompt of one head over its KV head's keys
        one = run_gpu(snapkv, q[h:h + 1], k[h // g:h // g + 1], v[h // g:h // g + 1], w.pool_kind, w.p, w.C)
        assert len(set(oiq[h].cpu().numpy().tolist()) ^ set(one[3][0].tolist())) <= 4
    assert snapkv.snapkv_sync_timeouts() == 0


def _random_long_shapes(seed, count):
    import random
    rng = random.Random(seed)
    out = []
    for it in range(count):
        g = rng.choice([1, 1, 2, 4])
        Hkv = rng.choice([1, 2, 4])
        W = rng.choice([8, 16, 16, 32, 32, 64, 128, 160])
        n = rng.choice([4200, 8193, 9000, 12288, 16385, 17000, 20011, 33000])
        C = W + rng.choice([1, 64, max(1, n // 9), max(1, n // 2), n - 1])
        out.append(Workload(f"randomlong{seed}_{it}", Hq=Hkv * g, Hkv=Hkv, D=rng.choice([64, 128]), L=W + n, W=W,
                            pool_kind=rng.choice([0, 1]), p=rng.choice([1, 5, 7, 13]), C=C,
                            dtype=rng.choice(["bf16", "bf16", "f16", "f32"]), clusters=(2, 6),
                            radius=rng.choice([1, 4, 9]), seed=3000 + it))
    return out


@pytest.mark.parametrize("w", _random_long_shapes(11, 40), ids=lambda w: w.name)
def test_random_shapes_with_few_resident_workgroups(few_slots, w):
    """Shapes nobody picked by hand, with the plans counting 16 resident workgroups: most of them are longer than
    the single-read launch holds (a front of 4096-16384 keys and a rest; the kept logits with 8- and 16-row windows
    of one query head per KV head), some fit it, windows of 160 rows take two streaming passes; each against the
    oracle."""
    gpu_vs_oracle(few_slots, w)
    assert few_slots.snapkv_sync_timeouts() == 0


def test_callers_workspace_and_static_scratch_on_the_long_path(few_slots):
    """The forms that do not allocate take the same launches: a caller's workspace (sized by
    snapkv_workspace_bytes, which includes the kept logits of a 16-row window) and the library's static array."""
    snapkv = few_slots
    for kw in (dict(L=12000, Hq=4, Hkv=4, C=256), dict(L=20000, W=16, p=5, Hq=4, Hkv=4, C=200)):
        w = Workload("long_ws", **dict(BASE, **kw))
        case = workloads.generate(w, device="cuda")
        q, k, v = case["q_win"], case["k"], case["v"]
        ref = run_gpu(snapkv, q, k, v, w.pool_kind, w.p, w.C)
        nbytes = snapkv.snapkv_workspace_bytes(w.L, w.Hq, w.Hkv, w.D, w.W)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for _ in range(2):      # the second call finds the workspace as the first left it
            ok, ov = torch.zeros_like(ref[1]), torch.zeros_like(ref[2])
            oi = torch.full(ref[3].shape, -1, dtype=torch.int32, device="cuda")
            assert snapkv.snapkv_compress(q, k, v, w.pool_kind, w.p, w.C, ok, ov, oi, workspace=ws) == w.C
            torch.cuda.synchronize()
            assert np.array_equal(oi.cpu().numpy(), ref[3]) and torch.equal(ok, ref[1]) and torch.equal(ov, ref[2])
        assert nbytes <= snapkv.STATIC_SCRATCH_BYTES
        ok, ov = torch.zeros_like(ref[1]), torch.zeros_like(ref[2])
        oi = torch.full(ref[3].shape, -1, dtype=torch.int32, device="cuda")
        assert snapkv.snapkv_compress_static(q, k, v, w.pool_kind, w.p, w.C, ok, ov, oi) == w.C
        torch.cuda.synchronize()
        assert np.array_equal(oi.cpu().numpy(), ref[3]) and torch.equal(ok, ref[1]) and torch.equal(ov, ref[2])
    assert snapkv.snapkv_sync_timeouts() == 0


@pytest.mark.parametrize("scheme,kw", [
    (4, dict(L=12000, Hq=4, Hkv=4, C=256)),                           # front and rest, both through the table of layers
    (4, dict(L=20000, W=16, p=5, Hq=4, Hkv=4, C=200)),                # ... with the rest's kept logits
    (4, dict(L=11000, Hq=16, Hkv=4, C=300, D=64, dtype="f16")),       # grouped-query heads
    (1, dict(L=6000, Hq=8, Hkv=4, C=256)),                            # two streaming passes through the table
], ids=["front_rest", "kept_logits", "gqa_f16_d64", "streaming"])
def test_separately_allocated_layers_of_long_prompts(snapkv, scheme, kw):
    """Layers that are allocations of their own share the launches of the long-prompt path too: every layer
    equals its own call bit for bit, one of them is checked against the oracle."""
    snapkv.snapkv_set_scoring_scheme(scheme)
    try:
        w = Workload("long_sep", **dict(BASE, layers=3, **kw))
        cases = [workloads.generate(w, layer=l, device="cuda") for l in range(3)]
        pads = [torch.empty(3000 + 100 * l, device="cuda") for l in range(3)]       # keeps the allocations apart
        oks = [torch.zeros((w.Hkv, w.C, w.D), dtype=cases[0]["k"].dtype, device="cuda") for _ in range(3)]
        ovs = [torch.zeros_like(t) for t in oks]
        ois = [torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda") for _ in range(3)]
        snapkv.snapkv_profile_start(16)
        snapkv.snapkv_compress_layers([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                      w.pool_kind, w.p, w.C, oks, ovs, ois)
        _, runs = snapkv.snapkv_profile_stop()
        assert runs == 1, "the three layers were meant to share one run of launches"
        for l, c in enumerate(cases):
            ref = run_gpu(snapkv, c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C)
            assert np.array_equal(ois[l].cpu().numpy(), ref[3]), f"layer {l}"
            assert torch.equal(oks[l], ref[1]) and torch.equal(ovs[l], ref[2]), f"layer {l}"
        check_against_oracle(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ref[0], oks[2], ovs[2],
                             ois[2].cpu().numpy(), w.C, own_topk_exact=scheme != 1)
        assert snapkv.snapkv_sync_timeouts() == 0
        del pads
    finally:
        snapkv.snapkv_set_scoring_scheme(0)
