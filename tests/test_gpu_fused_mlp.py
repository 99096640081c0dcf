"""GPU tests of gg_fp8_grouped_gemm_swiglu: the first GEMM of an expert MLP with silu(gate) * up and the 1x128
quantiser in its epilogue.

Stage by stage against the oracle, each oracle stage fed with the GPU's previous stage (fed with the oracle's own H
the final bytes would differ wherever H differs in its last bit, about 1 % of the elements):
  H, the bf16 output of the plain grouped GEMM on the same inputs, against the oracle's GEMM (tolerance of gg_testlib);
  the fused kernel's activations against the oracle's silu(gate) * up of H (one bf16 ulp: fp32 evaluation);
  its bytes and scales against the oracle's quantiser of those activations, BIT FOR BIT;
and, because the fused kernel holds the same accumulators as the plain one and then does the arithmetic of the
separate activation kernel, all three outputs against gg_fp8_swiglu_quantize_rows(H), BIT FOR BIT.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc
from workloads import CONFIGS, WorkloadConfig, make_problem
from gg_testlib import assert_parity, assert_swiglu_act, bits_of, np_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def u16(t):
    return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def check_against_two_calls_and_oracle(p, variants=(-1,), kmajor=(False, True), guard=2, empirical=True):
    A, SA, B, SB, off = (p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    M, N, K = p["M_total"], p["N"], p["K"]
    inter = N // 2
    H = gg.grouped_gemm(A, SA, B, SB, off, C=torch.zeros((M, N), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    Hb = u16(H)
    ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
    lo, hi = int(p["group_offsets"][0]), int(p["group_offsets"][-1])     # the oracle returns the rows of the groups
    assert_parity(Hb[lo:hi], ref, empirical=empirical, what="H of the plain GEMM")
    A2_two, SA2_two, act_two = gg.swiglu_quantize_rows(H, want_act=True)
    torch.cuda.synchronize()
    A2_two, SA2_two, act_two = A2_two.cpu().numpy(), SA2_two.cpu().numpy(), u16(act_two)
    for km in kmajor:
        SAx = SA.t().contiguous() if km else SA
        for v in variants:
            A2 = torch.full((M + 2 * guard, inter), 0xA5, dtype=torch.uint8, device=DEV)
            act = torch.full((M + 2 * guard, inter), 0x7B7B, dtype=torch.int16, device=DEV).view(torch.bfloat16)
            nblk = inter // 128
            sbuf = torch.full((nblk * M + 64,), -7.0, dtype=torch.float32, device=DEV)
            SA2 = sbuf[32:32 + nblk * M].view((nblk, M) if km else (M, nblk))
            gg.grouped_gemm_swiglu(A, SAx, B, SB, off, A2=A2[guard:guard + M], SA2=SA2, act_out=act[guard:guard + M],
                                   variant=v, sa_kmajor=km)
            torch.cuda.synchronize()
            what = f"variant {v}, {'K-block-major' if km else 'row-major'} scales"
            a2, ac, sb = A2.cpu().numpy(), u16(act), sbuf.cpu().numpy()
            s2 = SA2.cpu().numpy()
            s2 = np.ascontiguousarray(s2.T) if km else s2
            # rows outside the groups and the guard rows keep their canaries
            for name, arr, can in (("A2", a2, 0xA5), ("act", ac, 0x7B7B)):
                assert (arr[:guard + lo] == can).all() and (arr[guard + hi:] == can).all(), f"{what}: {name} written outside the groups"
            assert (sb[:32] == -7.0).all() and (sb[32 + nblk * M:] == -7.0).all(), f"{what}: SA2 guard"
            assert (s2[:lo] == -7.0).all() and (s2[hi:] == -7.0).all(), f"{what}: SA2 written outside the groups"
            got_act, got_a2, got_s2 = ac[guard + lo:guard + hi], a2[guard + lo:guard + hi], s2[lo:hi]
            # against the oracle
            assert_swiglu_act(Hb[lo:hi], got_act)
            A2_ref, SA2_ref = orc.quantize_rows(got_act)
            assert np.array_equal(got_s2.view(np.uint32), SA2_ref.view(np.uint32)), f"{what}: scales differ from the oracle's"
            bad = np.argwhere(got_a2 != A2_ref)
            assert bad.size == 0, f"{what}: {len(bad)} bytes differ from the oracle's, first at {bad[0]}"
            # against the two-kernel sequence
            assert np.array_equal(got_act, act_two[lo:hi]), f"{what}: activations differ from the separate kernel's"
            assert np.array_equal(got_a2, A2_two[lo:hi]) and np.array_equal(got_s2.view(np.uint32), SA2_two[lo:hi].view(np.uint32)), what


@pytest.mark.parametrize("sizes,inter,K", [
    ([0, 1, 299, 128, 17], 128, 512),               # one column block; empty and one-row groups; shortest K loop
    ([700, 0, 1300, 37, 1800, 191], 1024, 1024),    # several tiles per workgroup (the K loop carries on into the next)
    ([5, 300, 64], 384, 1536),                      # three column blocks, odd number of scale groups
    ([193, 225, 257], 256, 768),                    # one row more than each tile height
    ([700, 0, 1300, 37, 600], 512, 640),            # an odd number of K blocks, several tiles per workgroup
    ([5, 300, 64], 128, 384),                       # three K blocks: the shortest K loop there is
])
def test_fused_equals_gemm_then_oracle_activation_bitwise(sizes, inter, K):
    cfg = WorkloadConfig("fused", 5000 + inter + K, len(sizes), K, 2 * inter, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    check_against_two_calls_and_oracle(p, variants=[-1] + FUSED_VARIANTS_TAKEN(K))


def FUSED_VARIANTS_TAKEN(K=512):
    """The tile variants that have a twin with the activation epilogue: the second kernel's plain ones; with an odd
    number of K blocks the 192-row one only."""
    names = ("192x256/1x8w/3s-rb",) if (K // 128) % 2 else ("192x256/1x8w/3s-rb", "224x256/1x8w/3s-rb", "256x256/1x8w/3s-rb")
    return [v for v in range(gg.num_variants()) if gg.variant_name(v) in names]


def test_fused_special_values_and_rows_outside_the_groups():
    """NaN and huge weights (the activation overflows to infinity), groups that do not cover the buffer."""
    sizes, inter, K = [40, 0, 150], 256, 512
    cfg = WorkloadConfig("fusedx", 5100, len(sizes), K, 2 * inter, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    p["B"] = p["B"].clone()
    p["SB"] = p["SB"].clone()
    p["B"][0, 3, 5] = 0x7F                      # NaN in gate column 3 of group 0
    p["B"][2, inter + 9, 7] = 0xFF              # NaN in up column 9 of group 2
    p["SB"][2, 1, :] = 1.0e19                   # gate block 1 and up block 1 of group 2: both projections are finite,
    p["SB"][2, 2 + 1, :] = 1.0e22               # their product is not: act = +-inf (or -0 where the gate is negative)
    p["SB"][0, 2 + 1, 0] = 1.0e30               # up block 1 of group 0: huge but finite products
    # the groups leave 7 rows before and 5 after untouched
    M = p["M_total"]
    pad = lambda t, fill: torch.cat([torch.full((7,) + tuple(t.shape[1:]), fill, dtype=t.dtype), t, torch.full((5,) + tuple(t.shape[1:]), fill, dtype=t.dtype)])
    p["A"], p["SA"] = pad(p["A"], 0x38), pad(p["SA"], 1.0)
    p["group_offsets"] = p["group_offsets"] + 7
    p["M_total"] = M + 12
    check_against_two_calls_and_oracle(p, variants=[-1] + FUSED_VARIANTS_TAKEN(), empirical=False)


def test_fused_rejects_what_it_cannot_take():
    z = lambda *s, dt=torch.uint8: torch.zeros(s, dtype=dt, device=DEV)
    off = torch.tensor([0, 4], dtype=torch.int32, device=DEV)
    for inter, K in [(192, 512), (128, 400), (128, 256)]:        # I % 128, K % 128, K <= 256
        with pytest.raises(gg.GGError) as e:
            gg.grouped_gemm_swiglu(z(4, K), z(4, -(-K // 128), dt=torch.float32), z(1, 2 * inter, K),
                                   z(1, -(-2 * inter // 128), -(-K // 128), dt=torch.float32), off)
        assert e.value.status == 3
    with pytest.raises(gg.GGError) as e:                          # a first-kernel variant
        gg.grouped_gemm_swiglu(z(4, 512), z(4, 4, dt=torch.float32), z(1, 256, 512), z(1, 2, 4, dt=torch.float32), off, variant=0)
    assert e.value.status == 3


def test_fused_full_size_equals_the_two_calls_bitwise():
    """gate_up at full size, in the launch configuration the chain benchmark times: against the two-kernel sequence
    (whose stages are checked against the oracle elsewhere), both storage orders of the scales."""
    p = make_problem(CONFIGS["gate_up"], device=DEV)
    A, SA, B, SB, off = (p[k] for k in ("A", "SA", "B", "SB", "group_offsets"))
    H = gg.grouped_gemm(A, SA, B, SB, off)
    A2r, S2r, actr = gg.swiglu_quantize_rows(H, want_act=True)
    for km in (False, True):
        A2, S2, act = gg.grouped_gemm_swiglu(A, SA.t().contiguous() if km else SA, B, SB, off, want_act=True, sa_kmajor=km)
        torch.cuda.synchronize()
        assert torch.equal(A2, A2r) and torch.equal(act.view(torch.int16), actr.view(torch.int16))
        assert torch.equal((S2.t().contiguous() if km else S2).view(torch.int32), S2r.view(torch.int32))
    # a sample of rows against the oracle, stage by stage
    rows = np.arange(0, p["M_total"], 97)
    ridx = torch.from_numpy(rows).to(DEV)
    act_s = u16(actr[ridx])
    assert_swiglu_act(u16(H[ridx]), act_s)
    A2o, S2o = orc.quantize_rows(act_s)
    assert np.array_equal(A2r.cpu().numpy()[rows], A2o) and np.array_equal(S2r.cpu().numpy()[rows].view(np.uint32), S2o.view(np.uint32))


def test_fused_at_the_largest_weight_offsets():
    """One expert with 2 * I * K = 2^30 bytes of weights (the entry point takes up to 2^31 - 1): the up rows start
    2^29 bytes after the gate rows, the largest 32-bit scalar offset the kernel forms.  Raw bytes, few rows."""
    rng = np.random.default_rng(5300)
    M, inter, K = 40, 32768, 16384
    KB, NB = K // 128, 2 * inter // 128
    A = rng.integers(0, 256, (M, K), dtype=np.uint8)
    A[(A & 0x7F) == 0x7F] = 0x35
    A[(A & 0x78) > 0x58] &= 0xBF
    B = torch.randint(0, 256, (1, 2 * inter, K), dtype=torch.uint8, generator=torch.Generator().manual_seed(5300))
    B[(B & 0x7F) == 0x7F] = 0x35
    B[(B & 0x78) > 0x50] &= 0xBF
    SA = rng.uniform(0.25, 4.0, (M, KB)).astype(np.float32)
    SB = rng.uniform(0.25, 4.0, (1, NB, KB)).astype(np.float32)
    off = np.array([0, M], dtype=np.int32)
    dA, dSA, dSB, doff = (torch.from_numpy(x).to(DEV) for x in (A, SA, SB, off))
    dB = B.to(DEV)
    H = gg.grouped_gemm(dA, dSA, dB, dSB, doff)
    A2r, S2r, actr = gg.swiglu_quantize_rows(H, want_act=True)
    A2, S2, act = gg.grouped_gemm_swiglu(dA, dSA, dB, dSB, doff, want_act=True)
    torch.cuda.synchronize()
    assert torch.equal(A2, A2r) and torch.equal(S2.view(torch.int32), S2r.view(torch.int32))
    assert torch.equal(act.view(torch.int16), actr.view(torch.int16))
    # the plain GEMM's H against the oracle on the columns at both ends of the two projections
    cols = np.r_[0:128, inter - 128:inter + 128, 2 * inter - 128:2 * inter]
    Bs = B[0, torch.from_numpy(cols)].numpy()[None]
    blk = cols[::128] // 128                                           # the 128-column blocks these columns come from
    ref = orc.grouped_gemm(A, SA, Bs, np.ascontiguousarray(SB[:, blk]), off, with_abs_sum=True)
    assert_parity(u16(H[:, torch.from_numpy(cols).to(DEV)]), ref, empirical=False, what="H at the ends of gate and up")
