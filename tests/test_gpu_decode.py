"""GPU parity of snapkv_decode_attention (through the C ABI) against the fp64 oracle.

Tolerance, from the kernel's arithmetic: logits are exact products accumulated in fp32, the
exponent argument carries one fp32 rounding at magnitude <= ~2^7 (2^-17 relative in the
exponential), the probabilities enter the last product split into two storage-type parts
(<= 2^-16 relative) and everything else is fp32.  The output is a convex combination of value rows, so
|gpu - oracle| <= 1e-4 * max|v| leaves a factor of about three over the sum of those terms; the lse
is compared to 1e-4 absolute.
"""
import numpy as np
import pytest
import torch

from oracle import decode_oracle as dec
from paper_2404_14469_amd import workloads
from paper_2404_14469_amd.workloads import DecodeWorkload

pytestmark = pytest.mark.gpu

TOL = 1e-4


def run(snapkv, w, case, with_lse=True):
    q, k, v, lens = case["q"], case["k_cache"], case["v_cache"], case["lens"]
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda") if with_lse else None
    snapkv.snapkv_decode_attention(q, k, v, w.S, out, lse, lens=lens)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy() if with_lse else None


def check(w, case, out, lse, seqs=None):
    seqs = list(range(w.B)) if seqs is None else seqs
    lens = case["lens"].cpu().tolist() if case["lens"] is not None else [w.S] * w.B
    for b in seqs:
        S = lens[b]
        qb = workloads.to_numpy_bits(case["q"][b:b + 1])
        kb = workloads.to_numpy_bits(case["k_cache"][b:b + 1, :, :S])
        vb = workloads.to_numpy_bits(case["v_cache"][b:b + 1, :, :S])
        want, want_lse = dec.decode_attention(qb, kb, vb)
        vmax = float(np.abs(dec.widen(vb)).max())
        err = np.abs(out[b] - want[0]).max()
        assert err <= TOL * vmax, (w.name, b, err, vmax)
        if lse is not None:
            assert np.abs(lse[b] - want_lse[0]).max() <= TOL, (w.name, b)


CASES = [
    DecodeWorkload("one_pair", B=1, Hq=4, Hkv=4, D=128, S=32, cap=32, seed=1),
    DecodeWorkload("one_row", B=2, Hq=2, Hkv=2, D=64, S=1, cap=8, seed=2),
    DecodeWorkload("ragged_tail", B=2, Hq=8, Hkv=8, D=128, S=1000, cap=1100, seed=3),       # S % 32 != 0, S < cap
    DecodeWorkload("gqa4", B=3, Hq=16, Hkv=4, D=128, S=777, cap=800, seed=4),
    DecodeWorkload("gqa8_d64", B=2, Hq=32, Hkv=4, D=64, S=1500, cap=1500, seed=5),
    DecodeWorkload("gqa16", B=1, Hq=32, Hkv=2, D=128, S=300, cap=512, seed=6),             # a full 16-row operand
    DecodeWorkload("split_keys", B=1, Hq=8, Hkv=8, D=128, S=6000, cap=6000, seed=7),        # keys split over workgroups
    DecodeWorkload("split_ragged", B=2, Hq=8, Hkv=2, D=128, S=5000, cap=5003, ragged=True, seed=8),
    DecodeWorkload("many_pairs_no_split", B=40, Hq=32, Hkv=32, D=128, S=200, cap=200, seed=9),
    DecodeWorkload("lens_mixed", B=6, Hq=8, Hkv=4, D=64, S=900, cap=901, ragged=True, seed=10),
    DecodeWorkload("f16", B=2, Hq=8, Hkv=4, D=128, S=1234, cap=1300, dtype="f16", seed=11),
    DecodeWorkload("f16_d64_split", B=1, Hq=4, Hkv=4, D=64, S=4100, cap=4100, dtype="f16", seed=12),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_decode_matches_oracle(snapkv, w):
    case = workloads.generate_decode(w, device="cuda")
    out, lse = run(snapkv, w, case)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    check(w, case, out, lse)


def test_lse_output_is_optional_and_results_repeat_bitwise(snapkv):
    w = CASES[6]
    case = workloads.generate_decode(w, device="cuda")
    a, _ = run(snapkv, w, case, with_lse=False)
    b, _ = run(snapkv, w, case)
    assert np.array_equal(a, b)


def test_row_order_does_not_matter(snapkv):
    """The property a compacted cache relies on: permuting the cache rows changes nothing beyond
    the rounding order of the sums."""
    w = DecodeWorkload("perm", B=1, Hq=8, Hkv=8, D=128, S=3000, cap=3000, seed=21)
    case = workloads.generate_decode(w, device="cuda")
    a, la = run(snapkv, w, case)
    perm = torch.randperm(w.S, generator=torch.Generator().manual_seed(5)).cuda()
    case2 = dict(case, k_cache=case["k_cache"][:, :, perm].contiguous(), v_cache=case["v_cache"][:, :, perm].contiguous())
    b, lb = run(snapkv, w, case2)
    vmax = float(case["v_cache"].float().abs().max())
    assert np.abs(a - b).max() <= TOL * vmax and np.abs(la - lb).max() <= TOL


def test_empty_sequence_and_length_clamp(snapkv):
    w = DecodeWorkload("empty", B=3, Hq=4, Hkv=2, D=64, S=50, cap=64, seed=22)
    case = workloads.generate_decode(w, device="cuda")
    case["lens"] = torch.tensor([0, 50, 1000], dtype=torch.int32, device="cuda")   # 1000 is clamped to cap
    case["k_cache"][2, :, 50:] = case["k_cache"][1, :, :14]                        # make the padding rows ordinary
    case["v_cache"][2, :, 50:] = case["v_cache"][1, :, :14]
    out, lse = run(snapkv, w, case)
    assert np.array_equal(out[0], np.zeros_like(out[0])) and np.isneginf(lse[0]).all()
    case_ok = dict(case, lens=torch.tensor([1, 50, 64], dtype=torch.int32, device="cuda"))
    check(w, case_ok, out, lse, seqs=[1, 2])


def test_compressed_cache_feeds_the_decoding_step(snapkv):
    """End to end over the boundary: compress a prompt, decode over the kept rows, and compare with
    the oracle's attention over the rows the oracle's compression keeps."""
    w = workloads.Workload("e2e", Hq=8, Hkv=4, D=128, L=3000, W=32, pool_kind=0, p=7, C=256, dtype="bf16",
                           clusters=(4, 4), radius=6, seed=31)
    case = workloads.generate(w, device="cuda")
    out_k, out_v, out_idx, kept = snapkv.compress(case["q_win"], case["k"], case["v"], w.pool_kind, w.p, w.C)
    q_new = case["q_win"][:, -1, :].contiguous().unsqueeze(0)                       # stands in for the next token's query
    out = torch.empty((1, w.Hq, w.D), dtype=torch.float32, device="cuda")
    snapkv.snapkv_decode_attention(q_new, out_k.unsqueeze(0), out_v.unsqueeze(0), kept, out)
    torch.cuda.synchronize()
    # the oracle attends to exactly the rows the GPU kept (gathered bit-exactly, checked elsewhere)
    want, _ = dec.decode_attention(workloads.to_numpy_bits(q_new), workloads.to_numpy_bits(out_k.unsqueeze(0)),
                                   workloads.to_numpy_bits(out_v.unsqueeze(0)))
    vmax = float(out_v.float().abs().max())
    assert np.abs(out.cpu().numpy() - want).max() <= TOL * vmax
    # and those rows are the oracle's selection, by the same rule as everywhere: scores within 1e-3, kept
    # positions exact outside the band around the threshold, the exact top-k of the GPU's own scores
    from parity import check_against_oracle
    sc = torch.empty((w.Hkv, w.n), dtype=torch.float32, device="cuda")
    snapkv.snapkv_pooled_scores(case["q_win"], case["k"], w.pool_kind, w.p, sc)
    torch.cuda.synchronize()
    check_against_oracle(case["q_win"], case["k"], case["v"], w.pool_kind, w.p, w.C, sc.cpu().numpy(), out_k, out_v,
                         out_idx.cpu().numpy(), kept)


def test_bad_arguments_are_refused(snapkv):
    w = DecodeWorkload("bad", B=1, Hq=4, Hkv=4, D=64, S=10, cap=16, seed=23)
    case = workloads.generate_decode(w, device="cuda")
    out = torch.empty((1, 4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_decode_attention(case["q"], case["k_cache"], case["v_cache"], 17, out)      # S > cap
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_decode_attention(case["q"], case["k_cache"], case["v_cache"], 0, out)
    qf = case["q"].float()
    with pytest.raises(snapkv.SnapKVError):
        snapkv.snapkv_decode_attention(qf, case["k_cache"].float(), case["v_cache"].float(), 10, out)   # fp32 storage
