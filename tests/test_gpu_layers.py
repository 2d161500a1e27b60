"""snapkv_compress_layers: several layers of one prompt in one call.  Every layer must get, bit for bit,
what its own snapkv_compress call gives (and so the oracle's result, checked on a sample), whether the
layers are slices of stacked tensors (the fast form: they pass through the kernels as one layer with more
heads) or separate allocations, and however many heads the stacked form ends up with."""
import numpy as np
import pytest
import torch

from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import Workload
from parity import check_against_oracle, run_gpu

pytestmark = pytest.mark.gpu


def layer_cases(n_layers, **kw):
    base = dict(L=3000, Hq=8, Hkv=4, D=128, W=32, pool_kind=0, p=7, C=256, dtype="bf16", clusters=(5, 5), radius=6,
                layers=n_layers, seed=4100)
    base.update(kw)
    w = Workload("layers", **base)
    return w, [workloads.generate(w, layer=l, device="cuda") for l in range(n_layers)]


def stacked(cases, name):
    return torch.stack([c[name] for c in cases]).contiguous()


def outputs(w, n_layers, dtype, stack=True):
    if stack:
        ok = torch.zeros((n_layers, w.Hkv, w.C, w.D), dtype=dtype, device="cuda")
        ov = torch.zeros_like(ok)
        oi = torch.full((n_layers, w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
        return list(ok), list(ov), list(oi)
    oks = [torch.zeros((w.Hkv, w.C, w.D), dtype=dtype, device="cuda") for _ in range(n_layers)]
    return oks, [torch.zeros_like(t) for t in oks], [torch.full((w.Hkv, w.C), -1, dtype=torch.int32, device="cuda")
                                                      for _ in range(n_layers)]


def compare(snapkv, w, cases, oks, ovs, ois, oracle_on=()):
    rows = min(w.C, w.L)
    for l, c in enumerate(cases):
        ref = run_gpu(snapkv, c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C)
        assert ref[4] == rows
        assert np.array_equal(ois[l].cpu().numpy()[:, :rows], ref[3][:, :rows]), f"layer {l}: kept positions"
        assert torch.equal(oks[l][:, :rows], ref[1][:, :rows]) and torch.equal(ovs[l][:, :rows], ref[2][:, :rows]), \
            f"layer {l}: rows"
        if l in oracle_on:
            check_against_oracle(c["q_win"], c["k"], c["v"], w.pool_kind, w.p, w.C, ref[0], oks[l], ovs[l],
                                 ois[l].cpu().numpy(), rows)


SHAPES = {
    "mha_w32": dict(n_layers=3),
    "gqa_avg_w16": dict(n_layers=4, Hq=16, Hkv=4, W=16, pool_kind=1, p=5, C=300, L=4100),
    "d64_f16": dict(n_layers=3, D=64, dtype="f16", C=200, L=2222),
    "f32_tiny": dict(n_layers=5, Hq=4, Hkv=4, D=64, dtype="f32", L=512, C=128),
    "w64_p13": dict(n_layers=2, W=64, p=13, C=512, L=5000),
    "many_heads": dict(n_layers=48, Hq=8, Hkv=8, L=1500, C=160),     # 384 heads: more than the chip keeps resident
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_stacked_layers_equal_single_calls(snapkv, name):
    kw = dict(SHAPES[name])
    n_layers = kw.pop("n_layers")
    w, cases = layer_cases(n_layers, **kw)
    q, k, v = stacked(cases, "q_win"), stacked(cases, "k"), stacked(cases, "v")
    oks, ovs, ois = outputs(w, n_layers, k.dtype)
    snapkv.snapkv_compress_layers(list(q), list(k), list(v), w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    stacked_cases = [dict(q_win=q[l], k=k[l], v=v[l]) for l in range(n_layers)]
    compare(snapkv, w, stacked_cases, oks, ovs, ois, oracle_on=(0, n_layers - 1) if n_layers <= 8 else (n_layers - 1,))
    assert snapkv.snapkv_sync_timeouts() == 0


def test_separate_and_partly_stacked_layers(snapkv):
    """Layers that do not lie behind one another run one by one inside the call; a list may mix both."""
    w, cases = layer_cases(4)
    oks, ovs, ois = outputs(w, 4, cases[0]["k"].dtype, stack=False)
    snapkv.snapkv_compress_layers([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                  w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    compare(snapkv, w, cases, oks, ovs, ois)
    # layers 0-1 stacked in all six tensors, layers 2-3 stacked inputs but separate outputs
    q, k, v = stacked(cases, "q_win"), stacked(cases, "k"), stacked(cases, "v")
    a_k, a_v, a_i = outputs(w, 2, k.dtype)
    b_k, b_v, b_i = outputs(w, 2, k.dtype, stack=False)
    snapkv.snapkv_compress_layers(list(q), list(k), list(v), w.pool_kind, w.p, w.C, a_k + b_k, a_v + b_v, a_i + b_i)
    torch.cuda.synchronize()
    compare(snapkv, w, cases, a_k + b_k, a_v + b_v, a_i + b_i)


def test_layers_that_fit_the_capacity_and_empty_list(snapkv):
    w, cases = layer_cases(3, L=200, C=256)
    q, k, v = stacked(cases, "q_win"), stacked(cases, "k"), stacked(cases, "v")
    oks, ovs, ois = outputs(w, 3, k.dtype)
    snapkv.snapkv_compress_layers(list(q), list(k), list(v), w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    for l in range(3):
        assert np.array_equal(ois[l].cpu().numpy()[:, :200], np.tile(np.arange(200), (w.Hkv, 1)))
        assert int(ois[l][:, 200:].max()) == -1                      # rows beyond the prompt are not written
        assert torch.equal(oks[l][:, :200], k[l]) and torch.equal(ovs[l][:, :200], v[l])
    snapkv.snapkv_compress_layers([], [], [], 0, 7, 64, [], [], [])


def test_bad_layer_is_refused_before_anything_runs(snapkv):
    w, cases = layer_cases(2)
    q, k, v = stacked(cases, "q_win"), stacked(cases, "k"), stacked(cases, "v")
    oks, ovs, ois = outputs(w, 2, k.dtype)
    for t in ois:
        t.fill_(-7)
    with pytest.raises(snapkv.SnapKVError):      # an even pooling width
        snapkv.snapkv_compress_layers(list(q), list(k), list(v), 0, 6, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    assert all(int(t.min()) == -7 and int(t.max()) == -7 for t in ois)


def test_many_separate_layers_more_heads_than_stay_resident(snapkv):
    """40 separately allocated layers: two runs through the table of layer addresses (at most 32 layers each), with
    more heads than the cooperative selection keeps resident."""
    w, cases = layer_cases(40, Hq=8, Hkv=8, L=1500, C=160)
    oks, ovs, ois = outputs(w, 40, cases[0]["k"].dtype, stack=False)
    snapkv.snapkv_compress_layers([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                  w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    compare(snapkv, w, cases, oks, ovs, ois, oracle_on=(0, 39))
    assert snapkv.snapkv_sync_timeouts() == 0


@pytest.mark.parametrize("name", ["gqa_avg_w16", "d64_f16", "w64_p13", "f32_tiny"])
def test_separate_layers_of_other_shapes(snapkv, name):
    """Grouped-query heads, 16-row windows, D = 64 (table of layers); W = 64 and fp32 (one by one inside the call)."""
    kw = dict(SHAPES[name])
    n_layers = kw.pop("n_layers")
    w, cases = layer_cases(n_layers, **kw)
    oks, ovs, ois = outputs(w, n_layers, cases[0]["k"].dtype, stack=False)
    snapkv.snapkv_compress_layers([c["q_win"] for c in cases], [c["k"] for c in cases], [c["v"] for c in cases],
                                  w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    compare(snapkv, w, cases, oks, ovs, ois, oracle_on=(n_layers - 1,))
    assert snapkv.snapkv_sync_timeouts() == 0


def _random_layer_shapes(seed, count):
    import random
    rng = random.Random(seed)
    out = []
    for it in range(count):
        g = rng.choice([1, 1, 2, 4])
        Hkv = rng.choice([1, 2, 4, 8])
        W = rng.choice([8, 16, 32, 32, 48, 64])
        n = rng.choice([300, 1000, 2049, 4100, 9000])
        out.append(dict(n_layers=rng.choice([2, 3, 5, 7]), Hq=Hkv * g, Hkv=Hkv, W=W, L=W + n, D=rng.choice([64, 128]),
                        dtype=rng.choice(["bf16", "f16", "f32"]), pool_kind=rng.choice([0, 1]), p=rng.choice([1, 5, 7, 13]),
                        C=W + rng.choice([1, max(1, n // 8), max(1, n // 2)]), seed=4200 + it,
                        mix=rng.choice(["separate", "separate", "stacked", "outputs_separate"])))
    return out


@pytest.mark.parametrize("kw", _random_layer_shapes(5, 24), ids=lambda kw: f"{kw['mix']}_{kw['seed']}")
def test_random_layer_lists(snapkv, kw):
    """Layer lists nobody picked by hand (separate allocations, stacked tensors, stacked inputs with separate outputs;
    head counts, windows, lengths, storage types): every layer equals its own call, the last one the oracle."""
    kw = dict(kw)
    n_layers, mix = kw.pop("n_layers"), kw.pop("mix")
    w, cases = layer_cases(n_layers, **kw)
    if mix == "separate":
        q, k, v = ([c[n] for c in cases] for n in ("q_win", "k", "v"))
        oks, ovs, ois = outputs(w, n_layers, cases[0]["k"].dtype, stack=False)
    else:
        q, k, v = (list(stacked(cases, n)) for n in ("q_win", "k", "v"))
        oks, ovs, ois = outputs(w, n_layers, cases[0]["k"].dtype, stack=mix == "stacked")
    snapkv.snapkv_compress_layers(q, k, v, w.pool_kind, w.p, w.C, oks, ovs, ois)
    torch.cuda.synchronize()
    compare(snapkv, w, [dict(q_win=a, k=b, v=c) for a, b, c in zip(q, k, v)], oks, ovs, ois, oracle_on=(n_layers - 1,))
    assert snapkv.snapkv_sync_timeouts() == 0
