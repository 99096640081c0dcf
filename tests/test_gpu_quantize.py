"""GPU parity of the row quantiser (bf16 rows -> e4m3 bytes + 1x128 scales, gathered into group order):
the HIP kernel through the C ABI against the oracle, BIT FOR BIT (bytes and fp32 scales: integer work).

Both sides take the rounding decisions in float32 with correctly rounded division, as the header states.
Inputs are seeded and synthetic.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_bits(x32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def run_gpu(xb: np.ndarray, src=None, M_total=None, guard=3):
    """Returns (A, SA) and checks that the guard rows around the outputs keep their canaries."""
    X = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(DEV)
    T, K = xb.shape
    M = len(src) if src is not None else (T if M_total is None else M_total)
    A_buf = torch.full((M + 2 * guard, K), 0xA5, dtype=torch.uint8, device=DEV)
    SA_buf = torch.full((M + 2 * guard, K // 128), -7.0, dtype=torch.float32, device=DEV)
    src_d = None if src is None else torch.from_numpy(np.asarray(src, dtype=np.int32)).to(DEV)
    A, SA = gg.quantize_rows(X, src_d, M_total=M, A=A_buf[guard:guard + M], SA=SA_buf[guard:guard + M])
    torch.cuda.synchronize()
    Ab, Sb = A_buf.cpu().numpy(), SA_buf.cpu().numpy()
    assert (Ab[:guard] == 0xA5).all() and (Ab[guard + M:] == 0xA5).all()
    assert (Sb[:guard] == -7.0).all() and (Sb[guard + M:] == -7.0).all()
    return Ab[guard:guard + M], Sb[guard:guard + M]


def check(xb, src=None, M_total=None):
    A, SA = run_gpu(xb, src, M_total)
    A_ref, SA_ref = orc.quantize_rows(xb, src, M_total)
    assert np.array_equal(SA.view(np.uint32), SA_ref.view(np.uint32)), "scales differ"
    bad = np.argwhere(A != A_ref)
    assert bad.size == 0, f"{len(bad)} bytes differ, first at {bad[0]}: gpu {A[tuple(bad[0])]:#x} oracle {A_ref[tuple(bad[0])]:#x}"


@pytest.mark.parametrize("T,K", [(1, 128), (3, 256), (67, 7168), (130, 2048), (5, 4224)])   # 4224 = 33 blocks: ragged last pass
def test_random_rows_bit_exact(T, K):
    rng = np.random.default_rng(1000 + T + K)
    x = (rng.normal(0, 1, (T, K)) * np.exp(rng.normal(0, 4, (T, 1)))).astype(np.float32)
    check(bf16_bits(x))


def test_every_bf16_value_as_input():
    # all 65536 bf16 patterns (NaNs, infinities, subnormals, both zeros), 128 per block in pattern order and shuffled
    bits = np.arange(65536, dtype=np.uint16)
    rng = np.random.default_rng(5)
    xb = np.stack([bits.reshape(2, 32768)[0], bits.reshape(2, 32768)[1], rng.permutation(bits)[:32768], rng.permutation(bits)[:32768]])
    check(xb)
    # the same without NaN/inf, so that ordinary blocks see every finite exponent next to each other
    fin = bits[(bits & 0x7F80) != 0x7F80]
    xb = rng.permutation(np.concatenate([fin, fin[:256 - fin.size % 256]]))[: (fin.size // 256) * 256].reshape(-1, 256)
    check(xb)


def test_ties_and_exact_codes():
    # blocks whose scale is a power of two and whose values are exact e4m3 codes or exact midpoints of two codes
    table = orc.e4m3_decode_table()
    pos = np.arange(0, 0x7E)
    mids = (table[pos] + table[pos + 1]) / 2                      # 126 midpoints; every one is exact in bf16? keep those
    keep = orc.f64_from_bf16_bits(orc.bf16_bits_from_f64(mids)) == mids
    vals = np.concatenate([mids[keep], -mids[keep], table[pos], -table[pos]])
    rows = []
    for j in (-20, -1, 0, 3, 60):
        for start in range(0, vals.size, 127):
            blk = np.zeros(128)
            chunk = vals[start:start + 127]
            blk[:chunk.size] = chunk
            blk[127] = 448.0                                      # pins the scale to 2^j
            rows.append(blk * 2.0 ** j)
    x = np.stack(rows)
    xb = orc.bf16_bits_from_f64(x)
    assert np.array_equal(orc.f64_from_bf16_bits(xb), x)
    A, SA = run_gpu(xb)
    A_ref, SA_ref = orc.quantize_rows(xb)
    assert np.array_equal(A, A_ref) and np.array_equal(SA, SA_ref)
    assert set(np.log2(SA.ravel()).tolist()) == {-20.0, -1.0, 0.0, 3.0, 60.0}


def test_gather_into_group_order_and_invalid_sources():
    rng = np.random.default_rng(9)
    T, K = 300, 512
    xb = bf16_bits(rng.normal(0, 3, (T, K)).astype(np.float32))
    expert = rng.integers(0, 8, size=T)
    src = np.argsort(expert, kind="stable")                       # rows sorted by group: what MoE routing produces
    check(xb, src)
    src2 = np.concatenate([src[:50], [-1, T, 2 ** 31 - 1, -2 ** 31], src[::-1][:40], src[:10]])
    check(xb, src2)
    check(xb, None, M_total=T + 5)                                # identity with more output rows than inputs
    check(xb, None, M_total=7)


def test_zero_rows_and_empty_calls():
    xb = np.zeros((4, 256), np.uint16)
    xb[1] = 0x8000                                                # minus zeros
    A, SA = run_gpu(xb)
    assert (SA == np.float32(2.0 ** -100) / np.float32(448.0)).all() and not A[0].any() and (A[1] == 0x80).all()
    X = torch.zeros((0, 256), dtype=torch.bfloat16, device=DEV)
    A, SA = gg.quantize_rows(X)
    assert A.shape == (0, 256) and SA.shape == (0, 2)


def test_feeds_the_gemm_like_the_oracle_quantiser_does():
    # quantise on the GPU, multiply on the GPU; the oracle does both on the CPU: identical bytes in, parity out
    from gg_testlib import assert_parity, bits_of
    rng = np.random.default_rng(21)
    sizes, N, K = [70, 0, 129], 256, 512
    M = sum(sizes)
    xb = bf16_bits(rng.normal(0, 1, (M, K)).astype(np.float32))
    wb = bf16_bits((rng.normal(0, 0.02, (len(sizes) * N, K))).astype(np.float32))
    A_ref, SA_ref = orc.quantize_rows(xb)
    Bq, SBrow = orc.quantize_rows(wb)                             # weights: 1x128 here, expanded to 128x128 below
    # make the weight scales constant over 128 rows by re-quantising with the block maximum (power-of-two safe path)
    SB = SBrow.reshape(len(sizes), N // 128, 128, K // 128).max(axis=2)
    w = orc.f64_from_bf16_bits(wb).reshape(len(sizes), N // 128, 128, K // 128, 128)
    y = np.clip(w / SB[:, :, None, :, None].astype(np.float64), -448, 448).astype(np.float32)
    B = orc.e4m3_encode_rne(y).reshape(len(sizes), N, K)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    ref = orc.grouped_gemm(A_ref, SA_ref, B, SB.astype(np.float32), off, with_abs_sum=True)
    X = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(DEV)
    A, SA = gg.quantize_rows(X)
    C = gg.grouped_gemm(A, SA, torch.from_numpy(B).to(DEV), torch.from_numpy(SB.astype(np.float32)).to(DEV),
                        torch.from_numpy(off).to(DEV))
    torch.cuda.synchronize()
    assert_parity(bits_of(C), ref, what="quantise + GEMM")


def test_full_size_rows_sampled():
    # gate_up's activation tensor: 8192 x 7168, gathered by a routing permutation; every 61st row against the oracle
    T, K = 8192, 7168
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    X = (torch.randn((T, K), generator=gen, device=DEV) * torch.exp(torch.randn((T, 1), generator=gen, device=DEV))).to(torch.bfloat16)
    rng = np.random.default_rng(78)
    src = rng.permutation(T).astype(np.int32)
    A, SA = gg.quantize_rows(X, torch.from_numpy(src).to(DEV))
    torch.cuda.synchronize()
    rows = np.arange(0, T, 61)
    xb = X.view(torch.int16).cpu().numpy().view(np.uint16)
    A_ref, SA_ref = orc.quantize_rows(xb, src[rows])
    assert np.array_equal(A.cpu().numpy()[rows], A_ref)
    assert np.array_equal(SA.cpu().numpy()[rows], SA_ref)
