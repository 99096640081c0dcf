"""One expert layer forward and backward through the library, every call against its oracle on the GPU's own inputs:
Y = X W^T (quantise rows -> grouped GEMM), dX = dY W (the same GEMM on the transposed weights, whose 128 x 128 scale
blocks transpose with them), dW = dY^T X (quantise along the tokens -> variable-K grouped GEMM).  Seeded, synthetic.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from gg_testlib import assert_parity, bits_of
from oracle import gg_oracle as orc
from workloads.quantize import quantize_b

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def test_expert_layer_forward_and_backward():
    gen = torch.Generator().manual_seed(77)
    rng = np.random.default_rng(77)
    G, T, N, K = 4, 1008, 256, 512
    sizes = np.array([300, 0, 513, 195])
    off_np = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    X = torch.randn((T, K), generator=gen).to(torch.bfloat16)
    dY = (torch.randn((T, N), generator=gen) * 0.02).to(torch.bfloat16)        # already in group order
    W = torch.randn((G, N, K), generator=gen) * 0.02
    qw = [quantize_b(W[g].clone()) for g in range(G)]
    qwt = [quantize_b(W[g].t().contiguous()) for g in range(G)]
    Wq, SW = torch.stack([q for q, _ in qw]), torch.stack([s for _, s in qw])
    Wtq, SWt = torch.stack([q for q, _ in qwt]), torch.stack([s for _, s in qwt])
    assert torch.equal(Wtq, Wq.transpose(1, 2)) and torch.equal(SWt, SW.transpose(1, 2))   # the blocks transpose with the weights
    src = torch.from_numpy(rng.permutation(T).astype(np.int32))
    d = lambda t: t.to(DEV)
    off = d(torch.from_numpy(off_np))

    A, SA = gg.quantize_rows(d(X), d(src))
    Y = gg.grouped_gemm(A, SA, d(Wq), d(SW), off)
    dA, SdA = gg.quantize_rows(d(dY))
    dX = gg.grouped_gemm(dA, SdA, d(Wtq.contiguous()), d(SWt.contiguous()), off)
    XT, SX = gg.quantize_cols(d(X), d(src))
    DYT, SDY = gg.quantize_cols(d(dY))
    dW = gg.grouped_gemm_wgrad(XT, SX, DYT, SDY, off)
    torch.cuda.synchronize()

    xb, dyb = bf16_bits(X), bf16_bits(dY)
    A_ref, SA_ref = orc.quantize_rows(xb, src.numpy())
    assert np.array_equal(A.cpu().numpy(), A_ref) and np.array_equal(SA.cpu().numpy(), SA_ref)
    ref = orc.grouped_gemm(A_ref, SA_ref, Wq.numpy(), SW.numpy(), off_np, with_abs_sum=True)
    assert_parity(bits_of(Y), ref, what="forward")
    dA_ref, SdA_ref = orc.quantize_rows(dyb)
    assert np.array_equal(dA.cpu().numpy(), dA_ref) and np.array_equal(SdA.cpu().numpy(), SdA_ref)
    ref = orc.grouped_gemm(dA_ref, SdA_ref, Wtq.contiguous().numpy(), SWt.contiguous().numpy(), off_np, with_abs_sum=True)
    assert_parity(bits_of(dX), ref, what="input gradient")
    XT_ref, SX_ref = orc.quantize_cols(xb, src.numpy())
    DYT_ref, SDY_ref = orc.quantize_cols(dyb)
    assert np.array_equal(XT.cpu().numpy(), XT_ref) and np.array_equal(DYT.cpu().numpy(), DYT_ref)
    assert np.array_equal(SX.cpu().numpy(), SX_ref) and np.array_equal(SDY.cpu().numpy(), SDY_ref)
    ref = orc.grouped_gemm_wgrad(XT_ref, SX_ref, DYT_ref, SDY_ref, off_np, with_abs_sum=True)
    got = dW.cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref["D"])
    assert np.all(err <= np.spacing(np.abs(ref["D"]).astype(np.float32)).astype(np.float64) + 2.0 ** -13 * ref["S"])
    assert np.all(got[1] == 0)
    # and the three results mean what they should: against the float64 products of the unquantised tensors, within
    # the quantisation error of two e4m3 operands (a few percent of the result's scale)
    Xg = X.float().numpy().astype(np.float64)[src.numpy()]
    for g in range(G):
        lo, hi = off_np[g], off_np[g + 1]
        if hi == lo:
            continue
        want = dY.float().numpy().astype(np.float64)[lo:hi].T @ Xg[lo:hi]
        assert np.abs(got[g] - want).max() <= 0.08 * np.abs(want).max()
