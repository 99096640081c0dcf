"""GPU parity of the column quantiser (gg_fp8_quantize_cols: bf16 token rows -> e4m3 [K, M_total] + one scale per
feature and block of 128 tokens, gathered into group order and transposed: the producer of the weight-gradient
GEMM's operands): the HIP kernel through the C ABI against the oracle, BIT FOR BIT (bytes and fp32 scales).

Both sides take the rounding decisions in float32 with correctly rounded division.  Inputs are seeded and synthetic.
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


def run_gpu(xb, src=None, M_total=None, guard=2):
    """Returns (XT, SX) and checks that the guard rows around the outputs keep their canaries."""
    X = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(DEV)
    T, K = xb.shape
    M = len(src) if src is not None else (T if M_total is None else M_total)
    MB = (M + 127) // 128
    XT_buf = torch.full((K + 2 * guard, M), 0xA5, dtype=torch.uint8, device=DEV)
    SX_buf = torch.full((MB + 2 * guard, K), -7.0, dtype=torch.float32, device=DEV)
    src_d = None if src is None else torch.from_numpy(np.asarray(src, dtype=np.int32)).to(DEV)
    gg.quantize_cols(X, src_d, M_total=M, XT=XT_buf[guard:guard + K], SX=SX_buf[guard:guard + MB])
    torch.cuda.synchronize()
    Xb, Sb = XT_buf.cpu().numpy(), SX_buf.cpu().numpy()
    assert (Xb[:guard] == 0xA5).all() and (Xb[guard + K:] == 0xA5).all()
    assert (Sb[:guard] == -7.0).all() and (Sb[guard + MB:] == -7.0).all()
    return Xb[guard:guard + K], Sb[guard:guard + MB]


def check(xb, src=None, M_total=None):
    XT, SX = run_gpu(xb, src, M_total)
    XT_ref, SX_ref = orc.quantize_cols(xb, src, M_total)
    assert np.array_equal(SX.view(np.uint32), SX_ref.view(np.uint32)), "scales differ"
    bad = np.argwhere(XT != XT_ref)
    assert bad.size == 0, f"{len(bad)} bytes differ, first at {bad[0]}: gpu {XT[tuple(bad[0])]:#x} oracle {XT_ref[tuple(bad[0])]:#x}"


@pytest.mark.parametrize("T,K", [(16, 64), (128, 128), (144, 192), (400, 7168), (1040, 2048), (2000, 320)])
def test_random_tokens_bit_exact(T, K):
    """Whole and partial last token blocks (T % 128 = 16, 0, 16, 16, 16, 80), one to 112 feature tiles, magnitudes over
    many binades from token to token (the block maximum is then one token's, the others land on small codes)."""
    rng = np.random.default_rng(2000 + T + K)
    x = (rng.normal(0, 1, (T, K)) * np.exp(rng.normal(0, 4, (T, 1)))).astype(np.float32)
    check(bf16_bits(x))


def test_every_bf16_value_as_input():
    # all 65536 bf16 patterns (NaNs, infinities, subnormals, both zeros) down the tokens of 64 features, in pattern
    # order and shuffled; then the finite ones alone, so that ordinary blocks see every exponent next to each other
    bits = np.arange(65536, dtype=np.uint16)
    rng = np.random.default_rng(6)
    cols = [bits[:32768], bits[32768:]] + [rng.permutation(bits)[:32768] for _ in range(62)]
    check(np.ascontiguousarray(np.stack(cols, axis=1)))
    fin = bits[(bits & 0x7F80) != 0x7F80]
    n = (fin.size // 128) * 128
    check(np.ascontiguousarray(np.stack([rng.permutation(fin)[:n] for _ in range(64)], axis=1)))


def test_gather_with_repeated_and_invalid_sources():
    rng = np.random.default_rng(7)
    T, K, M = 500, 256, 1008
    xb = bf16_bits(rng.normal(0, 1, (T, K)).astype(np.float32))
    src = rng.integers(-3, T + 3, M)           # some outside [0, T): rows of zeros; many rows taken more than once
    src[128:256] = -1                          # a whole token block of zeros: scales 2^-100 / 448, bytes 0
    check(xb, src)
    XT, SX = run_gpu(xb, src)
    assert np.all(XT[:, 128:256] == 0) and np.all(SX[1] == np.float32(2.0 ** -100) / np.float32(448.0))


def test_full_size_activations_sampled_features():
    """gate_up's activations as the weight-gradient GEMM takes them: 8192 tokens x 7168 features through a routing
    permutation; the GPU quantises all of it, the oracle 448 sampled features (features are independent)."""
    rng = np.random.default_rng(8)
    T, K = 8192, 7168
    X = (torch.randn((T, K), generator=torch.Generator().manual_seed(8), dtype=torch.float32)).to(torch.bfloat16)
    src = rng.permutation(T).astype(np.int32)
    XT, SX = gg.quantize_cols(X.to(DEV), torch.from_numpy(src).to(DEV))
    torch.cuda.synchronize()
    feats = np.sort(rng.choice(K, 448, replace=False))
    feats[0], feats[-1] = 0, K - 1
    xb = X.view(torch.int16).numpy().view(np.uint16)
    XT_ref, SX_ref = orc.quantize_cols(np.ascontiguousarray(xb[:, feats]), src)
    assert np.array_equal(XT.cpu().numpy()[feats], XT_ref) and np.array_equal(SX.cpu().numpy()[:, feats], SX_ref)


def test_quantised_operands_feed_the_weight_gradient_gemm():
    """The training-side chain: both operands from gg_fp8_quantize_cols, then gg_fp8_grouped_gemm_wgrad; the oracle
    takes the same two steps, fed with the GPU's bytes and scales (which are bit-equal to its own)."""
    rng = np.random.default_rng(9)
    T, N, K = 1200, 256, 512
    off = np.array([0, 130, 130, 777, 1200], dtype=np.int32)
    xb = bf16_bits(rng.normal(0, 1, (T, K)).astype(np.float32))
    yb = bf16_bits(rng.normal(0, 0.02, (T, N)).astype(np.float32))
    src = rng.permutation(T).astype(np.int32)
    dev = lambda a: torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(DEV)
    XT, SX = gg.quantize_cols(dev(xb), torch.from_numpy(src).to(DEV))
    DYT, SDY = gg.quantize_cols(dev(yb))
    dW = gg.grouped_gemm_wgrad(XT, SX, DYT, SDY, torch.from_numpy(off).to(DEV))
    torch.cuda.synchronize()
    XT_ref, SX_ref = orc.quantize_cols(xb, src)
    DYT_ref, SDY_ref = orc.quantize_cols(yb)
    assert np.array_equal(XT.cpu().numpy(), XT_ref) and np.array_equal(SX.cpu().numpy(), SX_ref)
    assert np.array_equal(DYT.cpu().numpy(), DYT_ref) and np.array_equal(SDY.cpu().numpy(), SDY_ref)
    ref = orc.grouped_gemm_wgrad(XT_ref, SX_ref, DYT_ref, SDY_ref, off, with_abs_sum=True)
    got = dW.cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref["D"])
    bound = np.spacing(np.abs(ref["D"]).astype(np.float32)).astype(np.float64) + 2.0 ** -13 * ref["S"]
    assert np.all(err <= bound) and np.all(got[1] == 0)
