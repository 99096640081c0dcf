"""Pins of oracle.grouped_gemm_wgrad (the variable-K grouped GEMM of training: dW^g = dY^g^T X^g).

The paper names training in its title and the kernels around the grouped GEMM in Sec. 4 but defines no layouts or
scale granularity for this operation, so the function is parity unpinned against the paper; what fixes it here is the
mathematics of the definition written in its docstring: exact rational arithmetic by pure-Python loops, its
reduction to the (pinned) forward definition of Sec. 2.1 when there is one group and the second operand's scales are
constant over 128 features, closed forms, and the invariants a group-wise contraction has.  No GPU.
"""
from fractions import Fraction

import numpy as np
import torch

from oracle import gg_oracle as orc


def torch_decode(u8):
    t = torch.from_numpy(np.ascontiguousarray(u8)).view(torch.float8_e4m3fn)
    return t.to(torch.float32).numpy().astype(np.float64)


def random_bytes(rng, shape):
    b = rng.integers(0, 256, size=shape, dtype=np.uint8)
    b[(b & 0x7F) == 0x7F] = 0x3A
    return b


def problem(rng, M_total, N, K, lo=0.25, hi=4.0):
    MB = -(-M_total // 128)
    XT, DYT = random_bytes(rng, (K, M_total)), random_bytes(rng, (N, M_total))
    SX = rng.uniform(lo, hi, size=(MB, K)).astype(np.float32)
    SDY = rng.uniform(lo, hi, size=(MB, N)).astype(np.float32)
    return XT, SX, DYT, SDY


def exact_wgrad(XT, SX, DYT, SDY, off):
    """dW as exact Fractions, token by token: no blocks are formed, a token's factor is looked up by token // 128."""
    K, N = XT.shape[0], DYT.shape[0]
    Xi = np.rint(torch_decode(XT) * 512).astype(np.int64).tolist()
    Yi = np.rint(torch_decode(DYT) * 512).astype(np.int64).tolist()
    out = {}
    for g in range(len(off) - 1):
        for n in range(N):
            for k in range(K):
                tot, tot_abs = Fraction(0), Fraction(0)
                for r in range(off[g], off[g + 1]):
                    s = Fraction(float(SDY[r // 128, n])) * Fraction(float(SX[r // 128, k]))
                    p = Fraction(Yi[n][r] * Xi[k][r], 1 << 18)
                    tot += s * p
                    tot_abs += abs(s * p)
                out[(g, n, k)] = (tot, tot_abs)
    return out


def test_wgrad_against_exact_rationals_with_groups_that_cut_through_scale_blocks():
    rng = np.random.default_rng(11)
    off = [0, 37, 37, 130, 291, 300, 304]                  # an empty group, groups inside one block, a boundary at 130
    XT, SX, DYT, SDY = problem(rng, 304, 3, 5)
    res = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    exact = exact_wgrad(XT, SX, DYT, SDY, off)
    assert res["D"].shape == (6, 3, 5)
    for (g, n, k), (tot, tot_abs) in exact.items():
        d = Fraction(float(res["D"][g, n, k]))
        assert abs(d - tot) <= 8 * Fraction(1, 1 << 52) * tot_abs + 0
        assert abs(Fraction(float(res["S"][g, n, k])) - tot_abs) <= 8 * Fraction(1, 1 << 52) * tot_abs
    assert np.all(res["D"][1] == 0) and np.all(res["W"][1] == 0)          # the empty group
    assert res["W"].dtype == np.float32 and np.array_equal(res["W"], res["D"].astype(np.float32))


def test_wgrad_with_one_group_is_the_forward_definition_with_the_roles_renamed():
    """G = 1 over all tokens, SX constant over each 128 features: dW[0] = the D of Sec. 2.1's definition with
    A := DYT (rows n, contraction index = token), B[0] := XT, SA[n, j] := SDY[j, n], SB[0, k/128, j] := SX[j, k] -- the same
    partial sums, the same factors, the same order, so the two oracles must agree bit for bit."""
    rng = np.random.default_rng(12)
    M_total, N, K = 384, 7, 256
    XT, SX, DYT, SDY = problem(rng, M_total, N, K)
    SXb = rng.uniform(0.25, 4.0, size=(K // 128, M_total // 128)).astype(np.float32)
    SX = np.ascontiguousarray(np.repeat(SXb, 128, axis=0).T)
    w = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, [0, M_total])
    f = orc.grouped_gemm(DYT, np.ascontiguousarray(SDY.T), XT[None], SXb[None], [0, N])
    assert np.array_equal(w["D"][0], f["D"])


def test_wgrad_closed_forms_linearity_and_sum_over_groups():
    M_total, N, K = 272, 4, 6
    off = [0, 5, 133, 133, 272]
    ones_x, ones_y = np.full((K, M_total), 0x38, np.uint8), np.full((N, M_total), 0x38, np.uint8)
    SX = np.full((3, K), 0.5, np.float32)
    SDY = np.full((3, N), 3.0, np.float32)
    w = orc.grouped_gemm_wgrad(ones_x, SX, ones_y, SDY, off)
    for g, m in enumerate(np.diff(off)):
        assert np.all(w["D"][g] == 1.5 * m)                               # alpha * beta * M^g
    # small integers and power-of-two scales: every intermediate is exact, the groups add up to the one-group result
    rng = np.random.default_rng(13)
    codes = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0], np.uint8)      # 0, 1, 2, 3, -1, -2
    XT, DYT = codes[rng.integers(0, 6, (K, M_total))], codes[rng.integers(0, 6, (N, M_total))]
    SX = (2.0 ** rng.integers(-3, 4, (3, K))).astype(np.float32)
    SDY = (2.0 ** rng.integers(-3, 4, (3, N))).astype(np.float32)
    parts = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off)["D"]
    whole = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, [0, M_total])["D"]
    assert np.array_equal(parts.sum(axis=0), whole[0])
    # the same result from dequantised matrices and a plain product per group
    xd = torch_decode(XT) * np.repeat(SX.T.astype(np.float64), 128, axis=1)[:, :M_total]
    yd = torch_decode(DYT) * np.repeat(SDY.T.astype(np.float64), 128, axis=1)[:, :M_total]
    for g in range(4):
        assert np.array_equal(parts[g], yd[:, off[g]:off[g + 1]] @ xd[:, off[g]:off[g + 1]].T)
    # doubling SDY doubles the result; negating the bytes of one feature row negates its column
    assert np.array_equal(orc.grouped_gemm_wgrad(XT, SX, DYT, 2 * SDY, off)["D"], 2 * parts)
    XTn = XT.copy()
    XTn[2] ^= 0x80
    neg = orc.grouped_gemm_wgrad(XTn, SX, DYT, SDY, off)["D"]
    assert np.array_equal(neg[:, :, 2], -parts[:, :, 2]) and np.array_equal(np.delete(neg, 2, axis=2), np.delete(parts, 2, axis=2))


def test_wgrad_tokens_outside_a_group_do_not_matter_not_even_nan_codes():
    rng = np.random.default_rng(14)
    M_total, off = 320, [16, 100, 100, 250]                # tokens [0,16) and [250,320) belong to nobody
    XT, SX, DYT, SDY = problem(rng, M_total, 3, 4)
    base = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off)["D"]
    XT2, DYT2 = XT.copy(), DYT.copy()
    XT2[:, :16], DYT2[:, 250:] = 0x7F, 0xFF                # NaN codes outside every group
    assert np.array_equal(orc.grouped_gemm_wgrad(XT2, SX, DYT2, SDY, off)["D"], base)
    # a NaN inside group 2 reaches exactly the outputs of its feature row, in that group only
    XT3 = XT.copy()
    XT3[1, 120] = 0x7F
    d = orc.grouped_gemm_wgrad(XT3, SX, DYT, SDY, off)["D"]
    assert np.all(np.isnan(d[2, :, 1])) and np.isnan(d).sum() == 3
    mask = np.ones_like(d, bool)
    mask[2, :, 1] = False
    assert np.array_equal(d[mask], base[mask])


def bf16_bits(x):
    return (torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().astype(np.int32) & 0xFFFF).astype(np.uint16)


def test_quantize_cols_is_quantize_rows_on_the_transposed_matrix():
    """Whole token blocks: feature k's blocks along the tokens are the blocks of row k of X^T, so the (pinned) row
    quantiser on the transposed, gathered matrix must give the same bytes and the same scales, bit for bit."""
    rng = np.random.default_rng(21)
    T, K, M = 300, 24, 256
    X = bf16_bits(rng.standard_normal((T, K)) * np.exp(rng.uniform(-6, 6, (T, 1))))
    X[7, 3], X[9, 5], X[200, 0] = 0x7FC0, 0x7F80, 0xFF80                 # a NaN and two infinities
    row_src = rng.integers(-2, T + 2, M)                                  # some indices outside [0, T): rows of zeros
    XT, SX = orc.quantize_cols(X, row_src)
    gathered = np.zeros((M, K), np.uint16)
    ok = (row_src >= 0) & (row_src < T)
    gathered[ok] = X[row_src[ok]]
    A, SA = orc.quantize_rows(np.ascontiguousarray(gathered.T))           # [K, M], [K, M / 128]
    assert XT.shape == (K, M) and SX.shape == (2, K)
    assert np.array_equal(XT, A) and np.array_equal(SX, SA.T)


def test_quantize_cols_partial_last_block_and_closed_form():
    rng = np.random.default_rng(22)
    T, K = 200, 8                                                          # 128 + 72 tokens
    X = bf16_bits(rng.standard_normal((T, K)))
    XT, SX = orc.quantize_cols(X)
    # the last block sees its 72 tokens only: the same as a whole block whose other 56 tokens are zeros
    Xz = np.zeros((256, K), np.uint16)
    Xz[:T] = X
    XTz, SXz = orc.quantize_cols(Xz)
    assert XT.shape == (K, T) and np.array_equal(XT, XTz[:, :T]) and np.array_equal(SX, SXz)
    assert np.all(XTz[:, T:] == 0)
    # e4m3 values times a power of two per feature come back as their codes, with scale 2^e * max|value| / 448
    codes = rng.integers(1, 0x7F, (128, K)).astype(np.uint8)
    codes[0] = 0x7E                                                        # every feature holds 448
    e = rng.integers(-5, 6, K)
    vals = orc.e4m3_decode(codes) * 2.0 ** e[None, :]
    XTc, SXc = orc.quantize_cols(bf16_bits(vals))
    assert np.array_equal(XTc, codes.T) and np.array_equal(SXc[0], (2.0 ** e).astype(np.float32))
