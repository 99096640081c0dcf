"""GPU tests of the second storage order of the activation scales (GG_SA_KMAJOR: SA [ceil(K/128), M_total]).

Table 1 of the paper fixes the shape of the scale tensor, not how it is stored; the library takes both orders.
The order changes addresses only, never arithmetic, so every result must equal the row-major one BIT FOR BIT;
one result per case is also compared with the oracle (which takes SA row-major: the transposition is done here,
in NumPy), so that the tests do not only compare the library with itself.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc
from workloads import CONFIGS, WorkloadConfig, make_problem
from gg_testlib import assert_parity, bits_of, np_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CANARY = 0x7B7B


def canary(M, N):
    return torch.full((M, N), CANARY, dtype=torch.int16, device=DEV).view(torch.bfloat16)


def raw_ragged_problem(rng, sizes, N, K):
    sizes = np.asarray(sizes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    M, G = int(off[-1]), len(sizes)
    KB, NB = -(-K // 128), -(-N // 128)
    A = rng.integers(0, 256, (M, K), dtype=np.uint8)
    B = rng.integers(0, 256, (G, N, K), dtype=np.uint8)
    A[(A & 0x7F) == 0x7F] = 0x35
    B[(B & 0x7F) == 0x7F] = 0x35
    A[(A & 0x78) > 0x58] &= 0xBF
    SA = rng.uniform(0.25, 4.0, (M, KB)).astype(np.float32)
    SB = rng.uniform(0.25, 4.0, (G, NB, KB)).astype(np.float32)
    return A, SA, B, SB, off


@pytest.mark.parametrize("sizes,N,K,quantised", [
    ([0, 1, 299, 128, 17], 256, 256, True),              # the tiny shape: empty and one-row groups
    ([700, 0, 1300, 37, 1800, 191], 2048, 1024, True),   # several tiles per workgroup, both kernels
    ([5, 300, 64], 512, 512, True),
    ([70, 0, 129, 5], 200, 208, False),                  # ragged N and K (first kernel only)
    ([17, 1, 140], 8, 16, False),
    ([64, 64], 648, 4112, False),
])
def test_kmajor_scales_every_variant_bitwise_equal_to_row_major(sizes, N, K, quantised):
    rng = np.random.default_rng(4000 + N + K)
    if quantised:
        cfg = WorkloadConfig("order", 4000 + N, len(sizes), K, N, 0, "custom", "latency")
        host = np_problem(make_problem(cfg, sizes=np.array(sizes)))
    else:
        host = raw_ragged_problem(rng, sizes, N, K)
    A, SA, B, SB, off = host
    M = A.shape[0]
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    dA, dSA, dB, dSB, doff = (torch.from_numpy(np.ascontiguousarray(x)).to(DEV) for x in host)
    # K-block-major copy inside a larger buffer with canaries either side (the kernels only read it; the canaries
    # are NaNs, so a scale fetched from outside the tensor for a VALID row would show in the result)
    KB = SA.shape[1]
    buf = torch.full((KB * M + 64,), float("nan"), dtype=torch.float32, device=DEV)
    SAk = buf[32:32 + KB * M].view(KB, M)
    SAk.copy_(dSA.t())
    ran = 0
    for v in [-1] + list(range(gg.num_variants())):
        C0, C1 = canary(M + 2, N), canary(M + 2, N)
        try:
            gg.grouped_gemm(dA, dSA, dB, dSB, doff, C=C0[:M], variant=v)
        except gg.GGError as e:
            assert e.status == 3 and v >= 0          # this variant does not take the shape, in either order
            with pytest.raises(gg.GGError):
                gg.grouped_gemm(dA, SAk, dB, dSB, doff, C=C1[:M], variant=v, sa_kmajor=True)
            continue
        gg.grouped_gemm(dA, SAk, dB, dSB, doff, C=C1[:M], variant=v, sa_kmajor=True)
        torch.cuda.synchronize()
        b0, b1 = bits_of(C0), bits_of(C1)
        assert np.array_equal(b0, b1), f"variant {v}: the storage order of SA changed the result"
        assert (b1[M:] == CANARY).all()
        if v < 0:
            assert_parity(b1[:M], ref, empirical=quantised, what=f"K-major N={N} K={K}")
        ran += 1
    assert ran >= 5


def test_kmajor_binary16_output_and_untrusted_offsets():
    rng = np.random.default_rng(4100)
    sizes, N, K = [100, 100, 100], 256, 512
    A, SA, B, SB, off = raw_ragged_problem(rng, sizes, N, K)
    M = A.shape[0]
    dA, dSA, dB, dSB = (torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB))
    SAk = dSA.t().contiguous()
    good = torch.from_numpy(off).to(DEV)
    c0 = gg.grouped_gemm(dA, dSA, dB, dSB, good, out_dtype=torch.float16)
    c1 = gg.grouped_gemm(dA, SAk, dB, dSB, good, out_dtype=torch.float16, sa_kmajor=True)
    torch.cuda.synchronize()
    assert torch.equal(c0.view(torch.int16), c1.view(torch.int16))
    # offsets that leave [0, M_total] or decrease: nothing outside C is written, and where the clamped groups do not
    # overlap the two orders still agree (both clamp the offsets the same way)
    for bad in ([-50, 100, 200, 5000], [0, 250, 100, 300], [290, 295, 300, 1 << 30]):
        boff = torch.tensor(bad, dtype=torch.int32, device=DEV)
        for v in (-1, 0, 3, 12):
            C0, C1 = canary(M + 4, N), canary(M + 4, N)
            gg.grouped_gemm(dA, dSA, dB, dSB, boff, C=C0[2:2 + M], variant=v)
            gg.grouped_gemm(dA, SAk, dB, dSB, boff, C=C1[2:2 + M], variant=v, sa_kmajor=True)
            torch.cuda.synchronize()
            b0, b1 = bits_of(C0), bits_of(C1)
            assert (b1[:2] == CANARY).all() and (b1[2 + M:] == CANARY).all()
            if bad[2] >= bad[1]:          # decreasing offsets make two groups claim the same rows: the last writer wins
                assert np.array_equal(b0, b1)


@pytest.mark.parametrize("sizes,N,K", [([5, 300, 64], 256, 512), ([130, 0, 1, 67], 200, 336), ([0, 0, 7], 512, 4096)])
def test_kmajor_pad_path_bitwise(sizes, N, K):
    rng = np.random.default_rng(4200 + K)
    A, SA, B, SB, off = raw_ragged_problem(rng, sizes, N, K)
    M = A.shape[0]
    dA, dSA, dB, dSB, doff = (torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    SAk = dSA.t().contiguous()
    C_free = gg.grouped_gemm(dA, SAk, dB, dSB, doff, sa_kmajor=True)
    A_pad0, SA_pad0, poff0 = gg.pad(dA, dSA, doff)
    A_pad, SA_pad, poff = gg.pad(dA, SAk, doff, sa_kmajor=True)
    torch.cuda.synchronize()
    m_pad = int(poff[-1].item())          # rows past the last padded group are not written
    assert torch.equal(poff, poff0) and torch.equal(A_pad[:m_pad], A_pad0[:m_pad])
    assert torch.equal(SA_pad[:, :m_pad].contiguous().view(torch.int32), SA_pad0[:m_pad].t().contiguous().view(torch.int32)), "padded scales differ between the orders"
    C_pad = gg.grouped_gemm_padded(A_pad, SA_pad, dB, dSB, poff, sa_kmajor=True)
    C_back = gg.unpad(C_pad, doff, poff, M)
    C_row = gg.grouped_gemm(dA, dSA, dB, dSB, doff)
    torch.cuda.synchronize()
    assert torch.equal(C_back.view(torch.int16), C_free.view(torch.int16))
    assert torch.equal(C_row.view(torch.int16), C_free.view(torch.int16))
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    assert_parity(bits_of(C_back), ref, empirical=False, what="K-major pad path")


def test_kmajor_row_kernels_write_the_transposed_scales():
    rng = np.random.default_rng(4300)
    T, K, guard = 150, 1024, 40
    x = (rng.normal(0, 1, (T, K)) * np.exp(rng.normal(0, 3, (T, 1)))).astype(np.float32)
    X = torch.from_numpy(x).to(torch.bfloat16).to(DEV)
    xb = X.cpu().view(torch.int16).numpy().view(np.uint16)
    src = rng.integers(-2, T + 2, 333).astype(np.int32)              # gather with repeats and invalid sources
    M, KB = len(src), K // 128
    buf = torch.full((KB * M + 2 * guard,), -7.0, dtype=torch.float32, device=DEV)
    SAk = buf[guard:guard + KB * M].view(KB, M)
    A_k, _ = gg.quantize_rows(X, torch.from_numpy(src).to(DEV), SA=SAk, sa_kmajor=True)
    torch.cuda.synchronize()
    A_ref, SA_ref = orc.quantize_rows(xb, src, None)
    assert np.array_equal(A_k.cpu().numpy(), A_ref)
    assert np.array_equal(SAk.cpu().numpy().view(np.uint32), np.ascontiguousarray(SA_ref.T).view(np.uint32))
    b = buf.cpu().numpy()
    assert (b[:guard] == -7.0).all() and (b[guard + KB * M:] == -7.0).all()

    # the activation kernel
    Mh, I = 131, 640
    h = (rng.normal(0, 2, (Mh, 2 * I))).astype(np.float32)
    H = torch.from_numpy(h).to(torch.bfloat16).to(DEV)
    hb = H.cpu().view(torch.int16).numpy().view(np.uint16)
    IB = I // 128
    buf = torch.full((IB * Mh + 2 * guard,), -7.0, dtype=torch.float32, device=DEV)
    Sk = buf[guard:guard + IB * Mh].view(IB, Mh)
    A2, _, act = gg.swiglu_quantize_rows(H, SA=Sk, want_act=True, sa_kmajor=True)
    A2r, S2r, actr = gg.swiglu_quantize_rows(H, want_act=True)
    torch.cuda.synchronize()
    assert torch.equal(A2, A2r) and torch.equal(act.view(torch.int16), actr.view(torch.int16))
    assert torch.equal(Sk.view(torch.int32), S2r.t().contiguous().view(torch.int32))
    _, A_o, S_o = orc.swiglu_quantize_rows(hb)
    assert np.array_equal(A2.cpu().numpy(), A_o)
    assert np.array_equal(Sk.cpu().numpy().view(np.uint32), np.ascontiguousarray(S_o.T).view(np.uint32))
    b = buf.cpu().numpy()
    assert (b[:guard] == -7.0).all() and (b[guard + IB * Mh:] == -7.0).all()


@pytest.mark.parametrize("name", ["gate_up", "down", "decode"])
def test_kmajor_full_size_bitwise_equal_to_row_major(name):
    """At the sizes and in the launch configuration the benchmark times: both orders, automatic variant."""
    p = make_problem(CONFIGS[name], device=DEV)
    SAk = p["SA"].t().contiguous()
    c0 = gg.grouped_gemm(p["A"], p["SA"], p["B"], p["SB"], p["group_offsets"])
    c1 = gg.grouped_gemm(p["A"], SAk, p["B"], p["SB"], p["group_offsets"], sa_kmajor=True)
    torch.cuda.synchronize()
    assert torch.equal(c0.view(torch.int16), c1.view(torch.int16))
