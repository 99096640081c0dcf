"""Seeded random shapes through every entry point that takes them: the padding-free GEMM against the oracle, element
by element, and the identities that tie the other paths to it (K-block-major scales, pad path, fused activation
epilogue: all bit for bit).  The draws favour the edges: empty groups, groups of one row, group sizes next to tile
heights, N and K that are and are not multiples of 128 and 256."""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc
from gg_testlib import assert_parity, bits_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw(seed):
    rng = np.random.default_rng(seed)
    G = int(rng.integers(1, 7))
    edge = np.array([0, 1, 15, 16, 17, 127, 128, 129, 159, 160, 161, 191, 192, 193, 223, 224, 225, 255, 256, 257, 400])
    sizes = np.where(rng.random(G) < 0.6, rng.choice(edge, G), rng.integers(0, 500, G))
    N = int(rng.choice([8, 64, 128, 136, 256, 384, 512, 520, 768, 1024]))
    K = int(rng.choice([16, 128, 144, 256, 512, 768, 1024, 1040, 1536, 2048]))
    return rng, sizes, N, K


@pytest.mark.parametrize("seed", range(7000, 7016))
def test_random_shape_all_paths(seed):
    rng, sizes, N, K = draw(seed)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    M, G = int(off[-1]), len(sizes)
    KB, NB = -(-K // 128), -(-N // 128)
    A = rng.integers(0, 256, (max(M, 1), K), dtype=np.uint8)[:M]
    B = rng.integers(0, 256, (G, N, K), dtype=np.uint8)
    A[(A & 0x7F) == 0x7F] = 0x35
    B[(B & 0x7F) == 0x7F] = 0x35
    A[(A & 0x78) > 0x58] &= 0xBF                 # moderate magnitudes: finite bf16 results with scales up to 4
    B[(B & 0x78) > 0x50] &= 0xBF
    SA = rng.uniform(0.25, 4.0, (M, KB)).astype(np.float32)
    SB = rng.uniform(0.25, 4.0, (G, NB, KB)).astype(np.float32)
    dA, dSA, dB, dSB, doff = (torch.from_numpy(np.ascontiguousarray(x)).to(DEV) for x in (A, SA, B, SB, off))
    what = f"seed {seed}: sizes {sizes.tolist()} N={N} K={K}"
    C = gg.grouped_gemm(dA, dSA, dB, dSB, doff, C=torch.zeros((M, N), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    if M > 0:
        ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
        assert_parity(bits_of(C), ref, empirical=False, what=what)
    # K-block-major scales
    SAk = dSA.t().contiguous()
    Ck = gg.grouped_gemm(dA, SAk, dB, dSB, doff, C=torch.zeros((M, N), dtype=torch.bfloat16, device=DEV), sa_kmajor=True)
    # pad path, both orders
    outs = [Ck]
    for km in (False, True):
        A_pad, SA_pad, poff = gg.pad(dA, SAk if km else dSA, doff, sa_kmajor=km)
        C_pad = gg.grouped_gemm_padded(A_pad, SA_pad, dB, dSB, poff, sa_kmajor=km)
        outs.append(gg.unpad(C_pad, doff, poff, M, C=torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)))
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        assert torch.equal(o.view(torch.int16), C.view(torch.int16)), f"{what}: path {i} differs from the padding-free result"
    # the activation epilogue, where the shape allows it (and the plain GEMM adds the K blocks in the same order)
    if N % 256 == 0 and K % 128 == 0 and K > 256 and K % 8192 != 4096:
        A2r, S2r, actr = gg.swiglu_quantize_rows(C, want_act=True)
        for km in (False, True):
            A2, S2, act = gg.grouped_gemm_swiglu(dA, SAk if km else dSA, dB, dSB, doff, want_act=True, sa_kmajor=km,
                                                 A2=torch.zeros((M, N // 2), dtype=torch.uint8, device=DEV),
                                                 SA2=torch.zeros((N // 256, M) if km else (M, N // 256), dtype=torch.float32, device=DEV),
                                                 act_out=torch.zeros((M, N // 2), dtype=torch.bfloat16, device=DEV))
            torch.cuda.synchronize()
            # zero-filled outputs: rows of empty problems stay zero on both sides
            if M > 0:
                assert torch.equal(A2, A2r), f"{what}: fused bytes"
                assert torch.equal(act.view(torch.int16), actr.view(torch.int16)), f"{what}: fused activations"
                assert torch.equal((S2.t().contiguous() if km else S2).view(torch.int32), S2r.view(torch.int32)), f"{what}: fused scales"
