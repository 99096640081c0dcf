"""Pins of the CPU oracle against things that are not the oracle.

Each test fixes one part of oracle/gg_oracle.py to a value the paper prints, a
closed form, exact rational arithmetic, a library routine on a special case,
or an invariant, so that a dropped term, a swapped index or a wrong sign in the
oracle fails at least one of them.  Nothing here touches the GPU.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import gg_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# helpers that do NOT use the oracle
# ----------------------------------------------------------------------------
def torch_decode(u8: np.ndarray) -> np.ndarray:
    """e4m3fn bytes -> float64 through torch's own float8 type (library routine)."""
    t = torch.from_numpy(np.ascontiguousarray(u8)).view(torch.float8_e4m3fn)
    return t.to(torch.float32).numpy().astype(np.float64)


def random_bytes(rng, shape, allow_nan=False):
    b = rng.integers(0, 256, size=shape, dtype=np.uint8)
    if not allow_nan:
        b[(b & 0x7F) == 0x7F] = 0x3A     # replace the two NaN codes
    return b


def fraction_bf16_bits(x: Fraction) -> int:
    """bfloat16 bits of an exact rational, round-half-even, in rational arithmetic."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    a = -x if x < 0 else x
    # e = floor(log2 a)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    q = Fraction(2) ** (e - 7)
    n = round(a / q)                 # Python rounds exact halves to even
    v = n * q
    if v >= Fraction(2) ** 128:
        return sign | 0x7F80
    f = np.float32(float(v))         # v is a bfloat16 value: exact in float32
    assert Fraction(float(f)) == v
    return sign | int(np.array(f).view(np.uint32) >> 16)


def exact_reference(A, SA, B, SB, off):
    """D as exact Fractions by pure-Python loops over the definition (Table 1)."""
    G = len(off) - 1
    K, N = A.shape[1], B.shape[1]
    KB = -(-K // 128)
    Ai = np.rint(torch_decode(A) * 512).astype(np.int64).tolist()
    Bi = np.rint(torch_decode(B) * 512).astype(np.int64).tolist()
    out = {}
    for g in range(G):
        for r in range(off[g], off[g + 1]):
            for n in range(N):
                total = Fraction(0)
                tot_abs = Fraction(0)
                for kb in range(KB):
                    acc = 0
                    acc_abs = 0
                    ar, bn = Ai[r], Bi[g][n]
                    for k in range(kb * 128, min(K, kb * 128 + 128)):
                        p = ar[k] * bn[k]
                        acc += p
                        acc_abs += abs(p)
                    s = Fraction(float(SA[r, kb])) * Fraction(float(SB[g, n // 128, kb]))
                    total += s * Fraction(acc, 1 << 18)
                    tot_abs += abs(s) * Fraction(acc_abs, 1 << 18)
                out[(r, n)] = (total, tot_abs)
    return out


def small_problem(rng, sizes, N, K, scale_lo=0.25, scale_hi=4.0):
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    M, G = int(off[-1]), len(sizes)
    KB, NB = -(-K // 128), -(-N // 128)
    A = random_bytes(rng, (M, K))
    B = random_bytes(rng, (G, N, K))
    SA = rng.uniform(scale_lo, scale_hi, size=(M, KB)).astype(np.float32)
    SB = rng.uniform(scale_lo, scale_hi, size=(G, NB, KB)).astype(np.float32)
    return A, SA, B, SB, off


# ----------------------------------------------------------------------------
# P1  number formats
# ----------------------------------------------------------------------------
def test_e4m3_table_matches_library_and_spec_values():
    tab = orc.e4m3_decode_table()
    lib = torch_decode(np.arange(256, dtype=np.uint8))
    nan = np.isnan(lib)
    assert nan.sum() == 2 and nan[0x7F] and nan[0xFF]
    assert np.array_equal(np.isnan(tab), nan)
    assert np.array_equal(tab[~nan], lib[~nan])
    assert np.array_equal(np.signbit(tab[~nan]), np.signbit(lib[~nan]))
    # hand values from the OCP 8-bit float definition
    assert tab[0x00] == 0.0 and not np.signbit(tab[0x00])
    assert tab[0x80] == 0.0 and np.signbit(tab[0x80])
    assert tab[0x01] == 2.0 ** -9          # smallest subnormal
    assert tab[0x07] == 7 * 2.0 ** -9      # largest subnormal
    assert tab[0x08] == 2.0 ** -6          # smallest normal
    assert tab[0x38] == 1.0
    assert tab[0x3C] == 1.5
    assert tab[0x7E] == 448.0              # largest finite
    assert tab[0xFE] == -448.0
    assert tab[0x78] == 256.0              # exponent field 15 is NOT infinity


def test_bf16_rounding_matches_library_on_float32_inputs():
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 20000),
        np.array([0.0, -0.0, 1.0, -1.0, 3.3895314e38, -3.4e38, 1e-40, -1e-45, 9.18e-41,
                  np.inf, -np.inf], dtype=np.float32),
    ]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = orc.bf16_bits_from_f64(x.astype(np.float64))
    assert np.array_equal(got, lib)


def test_bf16_rounding_hand_values_and_single_step():
    b = orc.bf16_bits_from_f64
    one = 0x3F80
    assert b(np.array([1.0]))[0] == one
    assert b(np.array([1 + 2.0 ** -8]))[0] == one               # tie -> even (down)
    assert b(np.array([1 + 3 * 2.0 ** -8]))[0] == one + 2       # tie -> even (up) = 1 + 2^-6
    assert b(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == one + 1   # just above the tie
    # double rounding trap: 1 + 2^-8 + 2^-30 rounds to 1+2^-8 in float32 first (then ties to 1.0);
    # a single rounding step must go up.
    assert b(np.array([1 + 2.0 ** -8 + 2.0 ** -30]))[0] == one + 1
    assert b(np.array([np.nan]))[0] == 0x7FC0
    assert b(np.array([-0.0]))[0] == 0x8000
    assert b(np.array([2.0 ** 128]))[0] == 0x7F80
    big = (2 - 2.0 ** -7) * 2.0 ** 127                          # largest bf16
    assert b(np.array([big]))[0] == 0x7F7F
    assert b(np.array([(2 - 2.0 ** -8) * 2.0 ** 127]))[0] == 0x7F80   # tie at the top -> inf (even)
    assert b(np.array([2.0 ** -133]))[0] == 0x0001              # smallest subnormal
    assert b(np.array([2.0 ** -134]))[0] == 0x0000              # tie to even (0)
    assert b(np.array([-3 * 2.0 ** -134]))[0] == 0x8002
    # round trip
    bits = np.arange(0, 0x7F80, 37, dtype=np.uint16)
    assert np.array_equal(b(orc.f64_from_bf16_bits(bits)), bits)
    assert orc.bf16_ulp(np.array([1.0, 1.99, 2.0, 0.0]))[:3].tolist() == [2.0 ** -7, 2.0 ** -7, 2.0 ** -6]


def test_bf16_rounding_against_exact_rationals():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(3000) * 10.0 ** rng.integers(-42, 39, 3000)
    got = orc.bf16_bits_from_f64(x)
    for xi, gi in zip(x, got):
        assert int(gi) == fraction_bf16_bits(Fraction(float(xi)))


# ----------------------------------------------------------------------------
# P2 / P3  the whole definition against exact arithmetic and against a
#          dequantise-then-matmul evaluation
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("sizes,N,K", [
    ([3, 0, 1, 2], 260, 384),     # NB=3 (ragged), KB=3: catches a transposed SB index
    ([2, 2], 130, 200),           # ragged K block (ceil semantics of Table 1)
])
def test_against_exact_rational_brute_force(sizes, N, K):
    rng = np.random.default_rng(3)
    A, SA, B, SB, off = small_problem(rng, sizes, N, K)
    res = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    ref = exact_reference(A, SA, B, SB, off.tolist())
    KB = -(-K // 128)
    assert res["D"].shape == (int(off[-1]), N)
    for i, r in enumerate(res["rows"]):
        for n in range(N):
            exact, exact_abs = ref[(int(r), n)]
            d = Fraction(float(res["D"][i, n]))
            # only the KB multiplies and KB adds of the outer loop round
            assert abs(d - exact) <= 2 * KB * Fraction(1, 1 << 52) * exact_abs
            assert abs(Fraction(float(res["S"][i, n])) - exact_abs) <= 2 * KB * Fraction(1, 1 << 52) * exact_abs
            assert int(res["C"][i, n]) == fraction_bf16_bits(exact)


def test_inner_sum_is_exact_integer_arithmetic():
    # scales all 1 and a single K block: D must equal the integer dot product / 2^18 exactly
    rng = np.random.default_rng(4)
    sizes, N, K = [7, 9], 128, 128
    A, SA, B, SB, off = small_problem(rng, sizes, N, K)
    SA[:] = 1
    SB[:] = 1
    res = orc.grouped_gemm(A, SA, B, SB, off)
    Ai = np.rint(torch_decode(A) * 512).astype(np.int64)
    Bi = np.rint(torch_decode(B) * 512).astype(np.int64)
    for g in range(2):
        want = (Ai[off[g]:off[g + 1]] @ Bi[g].T).astype(np.float64) / 2.0 ** 18
        assert np.array_equal(res["D"][off[g]:off[g + 1]], want)


def test_against_dequantise_then_matmul():
    rng = np.random.default_rng(5)
    sizes, N, K = [40, 0, 131, 1, 77], 384, 512
    A, SA, B, SB, off = small_problem(rng, sizes, N, K)
    res = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    A_deq = torch_decode(A) * np.repeat(SA.astype(np.float64), 128, axis=1)
    for g in range(len(sizes)):
        B_deq = torch_decode(B[g]) * np.repeat(np.repeat(SB[g].astype(np.float64), 128, axis=0), 128, axis=1)
        want = A_deq[off[g]:off[g + 1]] @ B_deq.T
        got = res["D"][off[g]:off[g + 1]]
        S = res["S"][off[g]:off[g + 1]]
        assert np.all(np.abs(got - want) <= 1e-12 * S)
    assert res["D"].shape[0] == sum(sizes)


# ----------------------------------------------------------------------------
# P4  padded formulation == padding-free formulation, bit for bit (Sec. 3.2)
# ----------------------------------------------------------------------------
def test_padded_equals_unpadded_bitwise():
    rng = np.random.default_rng(6)
    sizes, N, K = [130, 0, 1, 128, 253, 127], 256, 256
    A, SA, B, SB, off = small_problem(rng, sizes, N, K)
    direct = orc.grouped_gemm(A, SA, B, SB, off)
    A_pad, SA_pad, poff = orc.pad(A, SA, off)
    assert poff.tolist() == [0, 256, 256, 384, 512, 768, 896]
    assert A_pad.shape[0] == 896
    padded = orc.grouped_gemm(A_pad, SA_pad, B, SB, poff)
    # pad rows: zero inputs, zero outputs
    valid = np.zeros(896, bool)
    for g in range(len(sizes)):
        valid[poff[g]:poff[g] + sizes[g]] = True
    assert not A_pad[~valid].any() and not SA_pad[~valid].any()
    assert not padded["D"][~valid].any()
    C = orc.unpad(padded["C"], off, poff, int(off[-1]))
    D = orc.unpad(padded["D"], off, poff, int(off[-1]))
    assert np.array_equal(C, direct["C"])
    assert np.array_equal(D.view(np.uint64), direct["D"].view(np.uint64))


# ----------------------------------------------------------------------------
# P5  zero-row and one-row groups
# ----------------------------------------------------------------------------
def test_zero_row_groups_shift_nothing_and_one_row_is_a_gemv():
    rng = np.random.default_rng(7)
    N, K = 256, 384
    A, SA, B, SB, off = small_problem(rng, [0, 1, 0, 0, 5, 0], N, K)
    res = orc.grouped_gemm(A, SA, B, SB, off)
    assert res["group"].tolist() == [1, 4, 4, 4, 4, 4]
    # dropping the empty groups (and their B) changes nothing
    keep = [1, 4]
    res2 = orc.grouped_gemm(A, SA, B[keep], SB[keep], np.array([0, 1, 6]))
    assert np.array_equal(res["C"], res2["C"])
    # the one-row group is a matrix-vector product with B^1
    a = torch_decode(A[0]) * np.repeat(SA[0].astype(np.float64), 128)
    Bd = torch_decode(B[1]) * np.repeat(np.repeat(SB[1].astype(np.float64), 128, axis=0), 128, axis=1)
    want = Bd @ a
    assert np.allclose(res["D"][0], want, rtol=1e-12, atol=1e-9)
    # all groups empty: nothing is produced
    empty = orc.grouped_gemm(A[:0], SA[:0], B, SB, np.zeros(7, dtype=np.int64))
    assert empty["D"].shape == (0, N)


def test_rows_outside_the_groups_are_not_produced_and_row_subsets_agree():
    rng = np.random.default_rng(8)
    A, SA, B, SB, off = small_problem(rng, [4, 3], 128, 128)
    # groups cover rows [2, 9) of an 11-row buffer
    A2 = np.concatenate([random_bytes(rng, (2, 128)), A, random_bytes(rng, (2, 128))])
    SA2 = np.concatenate([np.ones((2, 1), np.float32), SA, np.ones((2, 1), np.float32)])
    res = orc.grouped_gemm(A2, SA2, B, SB, off + 2)
    assert res["rows"].tolist() == list(range(2, 9))
    base = orc.grouped_gemm(A, SA, B, SB, off)
    assert np.array_equal(res["C"], base["C"])
    sub = orc.grouped_gemm(A, SA, B, SB, off, rows=np.array([6, 0, 3]))
    assert np.array_equal(sub["C"], base["C"][[6, 0, 3]])
    assert sub["group"].tolist() == [1, 0, 0]
    with pytest.raises(AssertionError):
        orc.grouped_gemm(A2, SA2, B, SB, off + 2, rows=np.array([0]))


# ----------------------------------------------------------------------------
# P6  permuting the groups permutes the row blocks of C
# ----------------------------------------------------------------------------
def test_group_permutation():
    rng = np.random.default_rng(9)
    sizes = [5, 0, 130, 1]
    A, SA, B, SB, off = small_problem(rng, sizes, 256, 256)
    base = orc.grouped_gemm(A, SA, B, SB, off)
    perm = [2, 3, 0, 1]
    A_p = np.concatenate([A[off[g]:off[g + 1]] for g in perm])
    SA_p = np.concatenate([SA[off[g]:off[g + 1]] for g in perm])
    off_p = np.concatenate([[0], np.cumsum([sizes[g] for g in perm])])
    res = orc.grouped_gemm(A_p, SA_p, B[perm], SB[perm], off_p)
    want = np.concatenate([base["C"][off[g]:off[g + 1]] for g in perm])
    assert np.array_equal(res["C"], want)
    # and using the wrong group's weights must show (the test can see a mix-up)
    wrong = orc.grouped_gemm(A_p, SA_p, B, SB, off_p)
    assert not np.array_equal(wrong["C"], want)


# ----------------------------------------------------------------------------
# P7  the paper's residual-row store rule: worked example of App. B, Eq. 1-2
# ----------------------------------------------------------------------------
def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            vals[k] = tuple(int(x) for x in v) if len(v) > 1 else int(v[0])
    return vals


def test_two_phase_cover_worked_example():
    gold = _read_golden("app_b_two_phase_example.txt")
    c = orc.two_phase_cover(gold["M_g"], gold["block_M"])
    for key in ("res", "rows_desc", "phase1_tile", "phase1_group", "phase2_tile", "phase2_group"):
        assert c[key] == gold[key], key
    overlap = c["phase1_group"][1] - c["phase2_group"][0] + 1
    assert overlap == gold["overlap_rows"]
    # the figure caption's group of 381 rows: same residual, shifted by one more full block
    c2 = orc.two_phase_cover(381, 128)
    assert c2["res"] == 125 and c2["phase1_tile"] == c["phase1_tile"] and c2["phase2_tile"] == c["phase2_tile"]
    assert c2["phase1_group"] == (256, 319) and c2["phase2_group"] == (317, 380)


def test_two_phase_cover_properties_and_pool():
    assert orc.descriptor_pool(128) == [1, 2, 4, 8, 16, 32, 64, 128]     # Eq. 1: i = 0..7
    for block_M in (64, 128, 256):
        pool = set(orc.descriptor_pool(block_M))
        assert orc.two_phase_cover(3 * block_M, block_M) is None
        for res in range(1, block_M):
            M_g = 2 * block_M + res
            c = orc.two_phase_cover(M_g, block_M)
            p = c["rows_desc"]
            assert p in pool and p <= res < 2 * p
            written = set(range(c["phase1_group"][0], c["phase1_group"][1] + 1)) | \
                set(range(c["phase2_group"][0], c["phase2_group"][1] + 1))
            assert written == set(range(M_g - res, M_g))        # all residual rows, none beyond
            # both phases move tile row t to group row (M_g - res) + t
            assert c["phase1_group"][0] - c["phase1_tile"][0] == M_g - res
            assert c["phase2_group"][0] - c["phase2_tile"][0] == M_g - res
            assert c["phase2_tile"][1] == res - 1


# ----------------------------------------------------------------------------
# P8 / P9  closed forms and linearity
# ----------------------------------------------------------------------------
def test_all_ones_closed_form():
    N, K = 256, 640
    sizes = [3, 2]
    M = 5
    A = np.full((M, K), 0x38, np.uint8)          # 1.0
    B = np.full((2, N, K), 0x38, np.uint8)
    alpha, beta = np.float32(0.375), np.float32(1.25)
    SA = np.full((M, 5), alpha, np.float32)
    SB = np.full((2, 2, 5), beta, np.float32)
    res = orc.grouped_gemm(A, SA, B, SB, np.array([0, 3, 5]))
    assert np.all(res["D"] == K * float(alpha) * float(beta))


def test_single_nonzero_block_and_scale_indexing():
    rng = np.random.default_rng(10)
    N, K = 384, 512
    A, SA, B, SB, off = small_problem(rng, [4, 4], N, K)
    # zero every A byte outside K block 2  => D = sa[:,2] * sb[g, n//128, 2] * inner_2
    A[:, :256] = 0
    A[:, 384:] = 0
    res = orc.grouped_gemm(A, SA, B, SB, off)
    Ad, Bd = torch_decode(A), torch_decode(B)
    for g in range(2):
        inner = Ad[off[g]:off[g + 1], 256:384] @ Bd[g][:, 256:384].T
        sb = np.repeat(SB[g, :, 2].astype(np.float64), 128)
        want = (SA[off[g]:off[g + 1], 2].astype(np.float64)[:, None] * sb[None, :]) * inner
        assert np.array_equal(res["D"][off[g]:off[g + 1]], want)


def test_power_of_two_scales_and_small_integers_are_exact():
    rng = np.random.default_rng(11)
    N, K = 256, 384
    sizes = [9, 6]
    off = np.array([0, 9, 15])
    small = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0, 0xC4], np.uint8)   # 0, 1, 2, 3, -1, -2, -3
    A = small[rng.integers(0, 7, (15, K))]
    B = small[rng.integers(0, 7, (2, N, K))]
    SA = (2.0 ** rng.integers(-3, 4, (15, 3))).astype(np.float32)
    SB = (2.0 ** rng.integers(-3, 4, (2, 2, 3))).astype(np.float32)
    res = orc.grouped_gemm(A, SA, B, SB, off)
    vals = {0x00: 0, 0x38: 1, 0x40: 2, 0x44: 3, 0xB8: -1, 0xC0: -2, 0xC4: -3}
    lut = np.zeros(256, np.int64)
    for k, v in vals.items():
        lut[k] = v
    Ai, Bi = lut[A], lut[B]
    for g in range(2):
        want = np.zeros((sizes[g], N))
        for kb in range(3):
            inner = Ai[off[g]:off[g + 1], kb * 128:(kb + 1) * 128] @ Bi[g][:, kb * 128:(kb + 1) * 128].T
            want += inner * SA[off[g]:off[g + 1], kb][:, None] * np.repeat(SB[g, :, kb], 128)[None, :]
        assert np.array_equal(res["D"][off[g]:off[g + 1]], want)      # integers * 2^j: no rounding anywhere


def test_linearity_in_scales_and_sign():
    rng = np.random.default_rng(12)
    A, SA, B, SB, off = small_problem(rng, [6, 5], 256, 256)
    base = orc.grouped_gemm(A, SA, B, SB, off)
    dbl = orc.grouped_gemm(A, SA * np.float32(2), B, SB, off)
    assert np.array_equal(dbl["D"], 2 * base["D"])
    halfb = orc.grouped_gemm(A, SA, B, SB * np.float32(0.5), off)
    assert np.array_equal(halfb["D"], 0.5 * base["D"])
    A_neg = A.copy()
    A_neg[3] ^= 0x80                                            # flip the sign of every byte of row 3
    neg = orc.grouped_gemm(A_neg, SA, B, SB, off)
    assert np.array_equal(neg["D"][3], -base["D"][3])
    assert np.array_equal(np.delete(neg["D"], 3, 0), np.delete(base["D"], 3, 0))


def test_nan_propagates_only_along_its_row_and_column():
    rng = np.random.default_rng(13)
    A, SA, B, SB, off = small_problem(rng, [4, 4], 128, 256)
    A[2, 130] = 0x7F
    B[1, 5, 7] = 0xFF
    res = orc.grouped_gemm(A, SA, B, SB, off)
    nan = np.isnan(res["D"])
    want = np.zeros_like(nan)
    want[2, :] = True
    want[4:8, 5] = True
    assert np.array_equal(nan, want)
    assert np.all(res["C"][nan] == 0x7FC0)


# ------------------------------------------------------------------------------------------------------------
# the row quantiser (producer of A and SA) and its encoder
# ------------------------------------------------------------------------------------------------------------
def _torch_e4m3(y32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(y32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_encoder_round_trips_every_code_and_breaks_ties_to_even():
    table = orc.e4m3_decode_table()
    codes = np.arange(256, dtype=np.uint8)
    finite = ~np.isnan(table)
    # every finite code is a fixed point (minus zero keeps its sign bit)
    assert np.array_equal(orc.e4m3_encode_rne(table[finite].astype(np.float32)), codes[finite])
    # midpoints of neighbouring positive codes go to the even code; one float32 step to either side decides
    pos = np.arange(0, 0x7E, dtype=np.uint8)                       # 0x7E = 448 is the last finite code
    lo, hi = table[pos], table[pos + 1]
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.all(mid.astype(np.float64) == (lo + hi) / 2)         # exactly representable
    even = np.where(pos % 2 == 0, pos, pos + 1).astype(np.uint8)
    assert np.array_equal(orc.e4m3_encode_rne(mid), even)
    assert np.array_equal(orc.e4m3_encode_rne(-mid), even | 0x80)
    assert np.array_equal(orc.e4m3_encode_rne(np.nextafter(mid, np.float32(0))), pos)
    assert np.array_equal(orc.e4m3_encode_rne(np.nextafter(mid, np.float32(1e9))), pos + 1)
    # NaN of either sign -> 0x7F
    assert orc.e4m3_encode_rne(np.array([np.nan, -np.nan], np.float32)).tolist() == [0x7F, 0x7F]


def test_encoder_matches_the_library_cast_on_every_bf16_value_in_range_and_on_random_float32():
    bits = np.arange(65536, dtype=np.uint32)
    v = (bits << 16).view(np.float32)
    v = v[np.abs(v) <= 448.0]                                       # drops NaN, inf and out-of-range
    assert v.size > 30000
    assert np.array_equal(orc.e4m3_encode_rne(v), _torch_e4m3(v))
    rng = np.random.default_rng(7)
    y = np.concatenate([rng.uniform(-448, 448, 300000), rng.normal(0, 1, 300000),
                        rng.uniform(-2.0 ** -5, 2.0 ** -5, 200000), rng.uniform(-2.0 ** -9, 2.0 ** -9, 50000)]).astype(np.float32)
    assert np.array_equal(orc.e4m3_encode_rne(y), _torch_e4m3(y))


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_row_quantiser_matches_the_same_recipe_in_library_ops():
    rng = np.random.default_rng(11)
    T, K = 37, 512
    x = (rng.normal(0, 1, (T, K)) * np.exp(rng.normal(0, 3, (T, 1)))).astype(np.float32)
    x[3, 128:256] = 0.0
    xb = _bf16_bits(x)
    A, SA = orc.quantize_rows(xb)
    xt = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).float().view(T, K // 128, 128)
    amax = xt.abs().amax(dim=2).clamp_min(2.0 ** -100)
    scale = amax / 448.0
    inv = torch.full_like(amax, 448.0) / amax        # tensor / tensor: a true division (scalar / tensor multiplies by a reciprocal)
    q = (xt * inv[:, :, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).view(T, K)
    assert np.array_equal(SA, scale.numpy())
    assert np.array_equal(A, q.numpy())
    assert SA[3, 1] == np.float32(2.0 ** -100) / np.float32(448.0) and not A[3, 128:256].any()


def test_row_quantiser_closed_forms_and_error_bound():
    table = orc.e4m3_decode_table()
    rng = np.random.default_rng(12)
    # a block made of exact e4m3 values times 2^j, its largest magnitude 448 * 2^j: scale = 2^j, codes come back
    K = 384
    codes = rng.integers(0, 0x7F, size=(5, K)).astype(np.uint8) | (rng.integers(0, 2, size=(5, K)).astype(np.uint8) << 7)
    codes[:, ::128] = 0x7E                                           # 448 somewhere in every block
    j = np.array([-3, 0, 5], dtype=np.float64)                        # one exponent per K block
    x = table[codes].reshape(5, 3, 128) * (2.0 ** j)[None, :, None]
    xb = orc.bf16_bits_from_f64(x.reshape(5, K))
    assert np.array_equal(orc.f64_from_bf16_bits(xb), x.reshape(5, K))   # 4 significant bits: exact in bf16
    A, SA = orc.quantize_rows(xb)
    assert np.array_equal(SA, np.broadcast_to((2.0 ** j).astype(np.float32), (5, 3)))
    assert np.array_equal(A, codes)
    # generic data: the largest element of a block encodes to +-448, and dequantising is within half a step
    x = rng.normal(0, 1, (64, 256)).astype(np.float32)
    xb = _bf16_bits(x)
    xv = orc.f64_from_bf16_bits(xb)
    A, SA = orc.quantize_rows(xb)
    deq = table[A] * np.repeat(SA.astype(np.float64), 128, axis=1)
    top = np.abs(xv.reshape(64, 2, 128)).argmax(axis=2)
    for r in range(64):
        for kb in range(2):
            assert (A[r, kb * 128 + top[r, kb]] & 0x7F) == 0x7E
    step = np.maximum(np.abs(xv) * 2.0 ** -4, np.repeat(SA.astype(np.float64), 128, axis=1) * 2.0 ** -10)
    assert np.all(np.abs(deq - xv) <= step * (1 + 1e-6))
    assert np.all(np.sign(deq) * np.sign(xv) >= 0)


def test_row_quantiser_gather_invalid_sources_and_nan():
    rng = np.random.default_rng(13)
    T, K = 20, 256
    xb = _bf16_bits(rng.normal(0, 2, (T, K)).astype(np.float32))
    A0, SA0 = orc.quantize_rows(xb)
    src = np.array([5, 5, 0, 19, -1, 20, 7], dtype=np.int64)
    A, SA = orc.quantize_rows(xb, src)
    for r, s in enumerate(src):
        if 0 <= s < T:
            assert np.array_equal(A[r], A0[s]) and np.array_equal(SA[r], SA0[s])
        else:
            assert not A[r].any() and np.all(SA[r] == np.float32(2.0 ** -100) / np.float32(448.0))
    # a NaN stays a NaN code in its place; the rest of its block is quantised as if it were not there
    xn = xb.copy()
    xn[2, 130] = 0x7FC0
    An, SAn = orc.quantize_rows(xn)
    xz = xb.copy()
    xz[2, 130] = 0
    Az, SAz = orc.quantize_rows(xz)
    assert An[2, 130] == 0x7F
    Az[2, 130] = 0x7F
    assert np.array_equal(An, Az) and np.array_equal(SAn, SAz)


def test_swiglu_closed_forms_library_routine_and_half_order():
    rng = np.random.default_rng(31)
    g = rng.normal(0, 3, (9, 256)).astype(np.float32)
    u = rng.normal(0, 2, (9, 256)).astype(np.float32)
    gb, ub = _bf16_bits(g), _bf16_bits(u)
    gv, uv = orc.f64_from_bf16_bits(gb), orc.f64_from_bf16_bits(ub)
    act = orc.swiglu_rows(np.concatenate([gb, ub], axis=1))
    assert act.shape == (9, 256) and act.dtype == np.uint16
    # the library's silu in float64, rounded by the (separately pinned) bf16 rounding
    ref = torch.nn.functional.silu(torch.from_numpy(gv)).numpy() * uv
    assert np.array_equal(act, orc.bf16_bits_from_f64(ref))
    # halves: a zero gate kills the product whatever `up` is; a large gate passes `up * gate` through
    one = _bf16_bits(np.ones((1, 128), np.float32))
    zero = np.zeros((1, 128), np.uint16)
    big = _bf16_bits(np.full((1, 128), 64.0, np.float32))
    assert not (orc.swiglu_rows(np.concatenate([zero, big], axis=1)) & 0x7FFF).any()
    assert np.array_equal(orc.swiglu_rows(np.concatenate([big, one], axis=1)), big)          # silu(64) = 64 to 2^-90
    assert not (orc.swiglu_rows(np.concatenate([one, zero], axis=1)) & 0x7FFF).any()
    # silu(x) - silu(-x) = x, silu(-large) -> -0, no overflow warnings matter
    x = np.array([[0.5, 1.0, 3.0, 20.0]], dtype=np.float32)
    xb = _bf16_bits(x)
    ones = _bf16_bits(np.ones_like(x))
    pos = orc.f64_from_bf16_bits(orc.swiglu_rows(np.concatenate([xb, ones], axis=1)))
    neg = orc.f64_from_bf16_bits(orc.swiglu_rows(np.concatenate([xb | 0x8000, ones], axis=1)))
    assert np.allclose(pos - neg, x, rtol=2.0 ** -7)
    far = orc.swiglu_rows(np.concatenate([_bf16_bits(np.full((1, 4), -1000.0, np.float32)), ones], axis=1))
    assert not (far & 0x7FFF).any()
    # chained with the quantiser: exactly quantize_rows of the activation bits
    actb, A, SA = orc.swiglu_quantize_rows(np.concatenate([gb, ub], axis=1))
    A2, SA2 = orc.quantize_rows(actb)
    assert np.array_equal(actb, act) and np.array_equal(A, A2) and np.array_equal(SA, SA2)


def test_binary16_rounding_against_the_library_hand_values_and_exact_rationals():
    rng = np.random.default_rng(51)
    x = np.concatenate([rng.normal(0, 1, 200000), rng.normal(0, 300, 100000), rng.uniform(-7e4, 7e4, 100000),
                        rng.uniform(-2.0 ** -13, 2.0 ** -13, 100000), rng.uniform(-2.0 ** -24, 2.0 ** -24, 1000)])
    with np.errstate(over="ignore"):
        lib = x.astype(np.float16).view(np.uint16)               # NumPy converts double -> half in one RNE step
    assert np.array_equal(orc.f16_bits_from_f64(x), lib)
    # every binary16 pattern decodes like the library and is a fixed point of the rounding
    bits = np.arange(65536, dtype=np.uint16)
    dec = orc.f64_from_f16_bits(bits)
    libdec = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(dec), np.isnan(libdec)) and np.array_equal(dec[~np.isnan(dec)], libdec[~np.isnan(dec)])
    fin = ~np.isnan(dec)
    assert np.array_equal(orc.f16_bits_from_f64(dec[fin]), bits[fin])
    # hand values: ties to even, the overflow threshold, the subnormal grid, signed zero, NaN
    cases = {1.0: 0x3C00, 1.0 + 2.0 ** -11: 0x3C00, 1.0 + 3 * 2.0 ** -11: 0x3C02, 65504.0: 0x7BFF, 65519.99: 0x7BFF,
             65520.0: 0x7C00, 1e9: 0x7C00, -1e9: 0xFC00, 2.0 ** -24: 0x0001, 2.0 ** -25: 0x0000, 1.5 * 2.0 ** -24: 0x0002,
             2.0 ** -14: 0x0400, -0.0: 0x8000, np.inf: 0x7C00}
    for v, b in cases.items():
        assert int(orc.f16_bits_from_f64(np.array([v]))[0]) == b, (v, b)
    assert int(orc.f16_bits_from_f64(np.array([np.nan]))[0]) == 0x7E00
    # one step, not two: 1 + 2^-11 + 2^-30 is above the tie and must round up even though float32 would hide the excess
    assert int(orc.f16_bits_from_f64(np.array([1.0 + 2.0 ** -11 + 2.0 ** -30]))[0]) == 0x3C01
    # exact rationals: the result is the nearest representable value
    for v in rng.normal(0, 10, 300):
        got = Fraction(float(orc.f64_from_f16_bits(orc.f16_bits_from_f64(np.array([v])))[0]))
        ulp = Fraction(float(orc.f16_ulp(np.array([v]))[0]))
        assert abs(got - Fraction(float(v))) <= ulp / 2
    assert orc.f16_ulp(np.array([1.0, 1.9, 2.0, 1e-9, 0.0])).tolist() == [2.0 ** -10, 2.0 ** -10, 2.0 ** -9, 2.0 ** -24, 2.0 ** -24]


def test_grouped_gemm_binary16_output_is_the_same_sum_rounded_once():
    rng = np.random.default_rng(52)
    A = rng.integers(0, 0x7E, (9, 256), dtype=np.uint8)
    B = rng.integers(0, 0x7E, (2, 128, 256), dtype=np.uint8)
    SA = rng.uniform(0.5, 2, (9, 2)).astype(np.float32)
    SB = rng.uniform(0.5, 2, (2, 1, 2)).astype(np.float32)
    off = np.array([0, 4, 9])
    r1 = orc.grouped_gemm(A, SA, B, SB, off)
    r2 = orc.grouped_gemm(A, SA, B, SB, off, out="f16")
    assert np.array_equal(r1["D"], r2["D"])
    with np.errstate(over="ignore"):
        assert np.array_equal(r2["C"], r2["D"].astype(np.float16).view(np.uint16))
