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
from gg_testlib import assert_swiglu_act

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


# ------------------------------------------------------------------------------------------------------------
# the activation between the two GEMMs, fused with the quantiser
# ------------------------------------------------------------------------------------------------------------
def check_swiglu(hb: np.ndarray, min_equal=0.995):
    """act: within one bf16 ulp of the oracle's float64 value (fp32 evaluation on the GPU; a result next to a
    rounding boundary may fall on the other side) plus |gate * up| * 2^-126 (below gate = -87.3 the fp32 sigmoid, itself
    below 2^-126, is flushed to 0), NaNs in the same places; bytes and scales:
    bit-exact against the oracle's quantiser applied to the GPU's own act bits (integer work; the fp decision
    sits in act)."""
    H = torch.from_numpy(hb.view(np.int16)).view(torch.bfloat16).to(DEV)
    A, SA, act = gg.swiglu_quantize_rows(H, want_act=True)
    A2, SA2, none = gg.swiglu_quantize_rows(H)
    torch.cuda.synchronize()
    assert none is None
    actb = act.view(torch.int16).cpu().numpy().view(np.uint16)
    A, SA = A.cpu().numpy(), SA.cpu().numpy()
    assert np.array_equal(A, A2.cpu().numpy()) and np.array_equal(SA, SA2.cpu().numpy())
    assert_swiglu_act(hb, actb, min_equal)
    A_ref, SA_ref = orc.quantize_rows(actb)
    assert np.array_equal(SA.view(np.uint32), SA_ref.view(np.uint32))
    assert np.array_equal(A, A_ref)


@pytest.mark.parametrize("M,I", [(1, 128), (67, 2048), (5, 4224), (130, 256)])
def test_swiglu_quantize_random(M, I):
    rng = np.random.default_rng(2000 + M + I)
    h = (rng.normal(0, 2, (M, 2 * I)) * np.exp(rng.normal(0, 1, (M, 1)))).astype(np.float32)
    check_swiglu(bf16_bits(h))


def test_swiglu_special_values():
    vals = np.array([0.0, -0.0, 1.0, -1.0, 20.0, -20.0, 88.0, -88.0, 90.0, -90.0, 1000.0, -1000.0, 3e38, -3e38,
                     np.inf, -np.inf, np.nan, 1e-30, -1e-30, 1e-40, 0.5, -0.5], dtype=np.float32)
    g, u = np.meshgrid(vals, vals, indexing="ij")
    n = g.size
    pad = (-n) % 128
    gate = np.concatenate([g.ravel(), np.zeros(pad, np.float32)]).reshape(1, -1)
    up = np.concatenate([u.ravel(), np.zeros(pad, np.float32)]).reshape(1, -1)
    check_swiglu(bf16_bits(np.concatenate([gate, up], axis=1)))


def test_swiglu_full_size_sampled_rows():
    # gate_up's output tensor: 8192 rows x (2 x 2048)
    M, I = 8192, 2048
    gen = torch.Generator(device=DEV)
    gen.manual_seed(79)
    H = (torch.randn((M, 2 * I), generator=gen, device=DEV) * 1.7).to(torch.bfloat16)
    A, SA, act = gg.swiglu_quantize_rows(H, want_act=True)
    torch.cuda.synchronize()
    rows = np.arange(0, M, 53)
    hb = H.view(torch.int16).cpu().numpy().view(np.uint16)[rows]
    actb = act.view(torch.int16).cpu().numpy().view(np.uint16)[rows]
    ref_bits = orc.swiglu_rows(hb)
    got, ref = orc.f64_from_bf16_bits(actb), orc.f64_from_bf16_bits(ref_bits)
    assert np.all(np.abs(got - ref) <= orc.bf16_ulp(ref))
    assert np.mean(actb == ref_bits) >= 0.995
    A_ref, SA_ref = orc.quantize_rows(actb)
    assert np.array_equal(A.cpu().numpy()[rows], A_ref) and np.array_equal(SA.cpu().numpy()[rows], SA_ref)


def test_expert_mlp_chain_stage_by_stage():
    # tokens -> quantise (gathered by expert) -> GEMM (gate|up) -> activation + quantise -> GEMM (down), every
    # stage on the GPU, every stage checked against the oracle fed with the GPU's previous stage
    from gg_testlib import assert_parity, bits_of
    from workloads.quantize import quantize_b
    rng = np.random.default_rng(41)
    sizes, hidden, inter = [70, 0, 129, 5], 512, 256
    G, M = len(sizes), sum(sizes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    xb = bf16_bits(rng.normal(0, 1, (M + 9, hidden)).astype(np.float32))          # 9 tokens routed nowhere
    src = rng.permutation(M + 9)[:M].astype(np.int32)
    gen = torch.Generator().manual_seed(42)
    W1 = [quantize_b(torch.randn((2 * inter, hidden), generator=gen) * 0.05) for _ in range(G)]
    W2 = [quantize_b(torch.randn((hidden, inter), generator=gen) * 0.05) for _ in range(G)]
    B1, SB1 = torch.stack([w[0] for w in W1]), torch.stack([w[1] for w in W1])
    B2, SB2 = torch.stack([w[0] for w in W2]), torch.stack([w[1] for w in W2])
    off_d = torch.from_numpy(off).to(DEV)
    X = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(DEV)

    A1, SA1 = gg.quantize_rows(X, torch.from_numpy(src).to(DEV))
    H = gg.grouped_gemm(A1, SA1, B1.to(DEV), SB1.to(DEV), off_d)
    A2, SA2, _ = gg.swiglu_quantize_rows(H)
    Y = gg.grouped_gemm(A2, SA2, B2.to(DEV), SB2.to(DEV), off_d)
    torch.cuda.synchronize()

    A1_ref, SA1_ref = orc.quantize_rows(xb, src)
    assert np.array_equal(A1.cpu().numpy(), A1_ref) and np.array_equal(SA1.cpu().numpy(), SA1_ref)
    ref1 = orc.grouped_gemm(A1_ref, SA1_ref, B1.numpy(), SB1.numpy(), off, with_abs_sum=True)
    assert_parity(bits_of(H), ref1, what="first GEMM of the chain")
    hb = bits_of(H)
    act_ref = orc.swiglu_rows(hb)
    A2_h, SA2_h = A2.cpu().numpy(), SA2.cpu().numpy()
    # the activation is not returned here: check it through the dequantised operand, half a quantisation step wide
    deq = orc.e4m3_decode_table()[A2_h] * np.repeat(SA2_h.astype(np.float64), 128, axis=1)
    actv = orc.f64_from_bf16_bits(act_ref)
    step = np.maximum(np.abs(actv) * 2.0 ** -4, np.repeat(SA2_h.astype(np.float64), 128, axis=1) * 2.0 ** -10)
    assert np.all(np.abs(deq - actv) <= step * 1.001 + orc.bf16_ulp(actv))
    ref2 = orc.grouped_gemm(A2_h, SA2_h, B2.numpy(), SB2.numpy(), off, with_abs_sum=True)
    assert_parity(bits_of(Y), ref2, what="second GEMM of the chain")
