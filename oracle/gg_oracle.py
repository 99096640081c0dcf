"""CPU oracle for the block-scaled FP8 grouped GEMM.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP library is measured against.  It is plain
NumPy in float64, shares no code, table or helper with the HIP path, and must
only be imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product never routes through it.

What it computes (paper Sec. 2.1, Table 1; 1x128 scaling of A and 128x128
scaling of B as stated right below Table 1):

    for every group g, every row r in [off[g], off[g+1]), every column n

        D[r, n] = sum_{kb ascending} ( SA[r, kb] * SB[g, n // 128, kb] )
                                     * ( sum_{k in K-block kb} dec(A[r, k]) * dec(B[g, n, k]) )
        C[r, n] = bf16_round_to_nearest_even( D[r, n] )

``dec`` is the OCP e4m3 ("fn") decoding.  Rows of C outside
[off[0], off[G]) are not produced.  N and K are shared by all groups, M^g is
per group (paragraph below Table 1); the output is a 2-byte float (App. A,
analysis of C^g) and this build fixes it to bfloat16.

Why a float64 matmul may serve as the inner step without being an
approximation: every e4m3 value is an integer multiple of 2^-9 of magnitude at
most 448, so every product is an integer multiple of 2^-18 below 2^18 and a sum
of 128 of them needs at most 43 significant bits.  The inner sum is therefore
exact in float64 in ANY summation order, and so is SA*SB (24+24 bits).  Only
the outer accumulation over kb rounds, and its order is fixed (ascending).

Every function here is pinned by tests/test_oracle_pins.py (exact rational
brute force, closed forms, the paper's worked example, the padded == unpadded
invariant of Sec. 3.2; the encoder and the row quantiser at the end of the file
against the library's float8 cast, round trips through the decode table and
hand-made ties; the activation against the library's silu and closed forms).  Two functions are "parity unpinned"
against the paper, which does not define them: grouped_gemm_wgrad (see the comment above it; pinned by
tests/test_oracle_wgrad_pins.py to the mathematics of its definition) and quantize_cols, the producer of its
operands (pinned there to quantize_rows, the same recipe on the transposed matrix).
"""
from __future__ import annotations

import numpy as np

SCALE_BLOCK = 128  # width of a scale block along K (A and B) and along N (B)  -- Sec. 2.1


# ----------------------------------------------------------------------------
# number formats
# ----------------------------------------------------------------------------
def e4m3_decode_table() -> np.ndarray:
    """float64[256]: value of every OCP e4m3fn byte, from the bit definition.

    1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent field 0 is
    subnormal (m * 2^-9); there is no infinity; S.1111.111 is NaN; the largest
    finite magnitude is 448.  (The paper only says "FP8"; e4m3 with max 448 is
    the reading fixed for this build.)
    """
    table = np.empty(256, dtype=np.float64)
    for byte in range(256):
        sign = -1.0 if (byte & 0x80) else 1.0
        e = (byte >> 3) & 0xF
        m = byte & 0x7
        if e == 0xF and m == 0x7:
            v = float("nan")
        elif e == 0:
            v = sign * m * 2.0 ** (-9)
        else:
            v = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
        table[byte] = v
    return table


_DEC = e4m3_decode_table()


def e4m3_decode(u8: np.ndarray) -> np.ndarray:
    """Decode an array of e4m3 bytes to float64."""
    u8 = np.asarray(u8)
    assert u8.dtype == np.uint8
    return _DEC[u8]


def bf16_bits_from_f64(x: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns of float64 values, ONE rounding step (RNE).

    bfloat16 = 1 sign, 8 exponent (bias 127), 7 mantissa bits.  The value is
    rounded on the bfloat16 grid directly (no detour through float32, which
    would round twice).  Overflow goes to +-inf, NaN becomes the canonical
    quiet NaN 0x7FC0, signed zeros are kept.
    """
    x = np.asarray(x, dtype=np.float64)
    sign = np.signbit(x)
    a = np.abs(x)
    nan = np.isnan(a)
    a = np.where(nan, 0.0, a)
    # exponent e with 2^e <= a < 2^(e+1); frexp gives a = f * 2^E, f in [0.5, 1)
    _, E = np.frexp(a)
    e = np.maximum(E.astype(np.int64) - 1, -126)  # subnormals share the grid of 2^-126
    quantum = np.ldexp(1.0, (e - 7).astype(np.int32))  # spacing of bf16 values in that binade
    with np.errstate(over="ignore", invalid="ignore"):
        ratio = a / quantum                  # exact: division by a power of two
        ratio = np.where(np.isinf(a), np.inf, ratio)
        r = np.rint(ratio) * quantum         # np.rint rounds half to even; product exact
    # r is now exactly a bfloat16 value (or 2^128 / inf => overflow); float32 holds it exactly
    with np.errstate(over="ignore"):
        f32 = r.astype(np.float32)
    bits = (f32.view(np.uint32) >> 16).astype(np.uint16)
    bits = np.where(sign, bits | np.uint16(0x8000), bits)
    bits = np.where(nan, np.uint16(0x7FC0), bits)
    return bits.astype(np.uint16)


def f64_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """float64 value of bfloat16 bit patterns (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 values in the binade that holds |x| (float64)."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    _, E = np.frexp(np.where(a == 0, 1.0, a))
    e = np.maximum(E.astype(np.int64) - 1, -126)
    e = np.where(a == 0, -126, e)
    return np.ldexp(1.0, (e - 7).astype(np.int32))


def f16_bits_from_f64(x: np.ndarray) -> np.ndarray:
    """uint16 IEEE binary16 bit patterns of float64 values, ONE rounding step (RNE): the other reading of the
    paper's "half-precision" output (App. A only fixes 2 bytes per element).

    binary16 = 1 sign, 5 exponent (bias 15), 10 mantissa bits; subnormals on the grid 2^-24; the largest finite
    value is 65504 and anything that rounds to 2^16 becomes +-inf.  NaN becomes 0x7E00, signed zeros are kept.
    """
    x = np.asarray(x, dtype=np.float64)
    sign = np.signbit(x)
    a = np.abs(x)
    nan = np.isnan(a)
    a = np.where(nan, 0.0, a)
    _, E = np.frexp(a)
    e = np.maximum(E.astype(np.int64) - 1, -14)          # subnormals share the grid of 2^-14
    quantum = np.ldexp(1.0, (e - 10).astype(np.int32))
    with np.errstate(over="ignore", invalid="ignore"):
        ratio = np.where(np.isinf(a), np.inf, a / quantum)
        r = np.rint(ratio) * quantum                     # exactly a binary16 value, or >= 2^16 (overflow)
    inf = r >= 2.0 ** 16
    r = np.where(inf, 0.0, r)
    m, E2 = np.frexp(r)                                  # r = m * 2^E2, m in [0.5, 1)
    e2 = E2.astype(np.int64) - 1
    normal = r >= 2.0 ** -14
    frac = np.where(normal, np.rint((2.0 * m - 1.0) * 1024.0), np.rint(r * 2.0 ** 24)).astype(np.int64)   # exact
    bits = np.where(normal, ((e2 + 15) << 10) | frac, frac)
    bits = np.where(inf, 0x7C00, bits)
    bits = np.where(sign, bits | 0x8000, bits)
    bits = np.where(nan, 0x7E00, bits)
    return bits.astype(np.uint16)


def f64_from_f16_bits(bits: np.ndarray) -> np.ndarray:
    """float64 value of binary16 bit patterns (exact), from the format's definition."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    sign = np.where(b & 0x8000, -1.0, 1.0)
    e = (b >> 10) & 0x1F
    m = (b & 0x3FF).astype(np.float64)
    with np.errstate(invalid="ignore"):
        v = np.where(e == 0, m * 2.0 ** -24, np.ldexp(1.0 + m / 1024.0, (e - 15).astype(np.int32)))
        v = np.where(e == 0x1F, np.where(m == 0, np.inf, np.nan), v)
    return sign * v


def f16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of binary16 values in the binade that holds |x| (float64); 2^-24 below 2^-14."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    _, E = np.frexp(np.where(a == 0, 1.0, a))
    e = np.maximum(E.astype(np.int64) - 1, -14)
    e = np.where(a == 0, -14, e)
    return np.ldexp(1.0, (e - 10).astype(np.int32))


# ----------------------------------------------------------------------------
# the operation
# ----------------------------------------------------------------------------
def _check_shapes(A, SA, B, SB, off, N, K):
    G = off.shape[0] - 1
    KB = -(-K // SCALE_BLOCK)
    NB = -(-N // SCALE_BLOCK)
    assert A.dtype == np.uint8 and A.ndim == 2 and A.shape[1] == K
    assert B.dtype == np.uint8 and B.shape == (G, N, K)
    assert SA.shape == (A.shape[0], KB)
    assert SB.shape == (G, NB, KB)
    return G, KB, NB


def grouped_gemm(A, SA, B, SB, group_offsets, rows=None, with_abs_sum=False, out="bf16"):
    """Block-scaled FP8 grouped GEMM by its definition (Sec. 2.1, Table 1).

    A   uint8 [M_total, K]   e4m3 bytes, groups concatenated along rows
    SA  float [M_total, ceil(K/128)]     one scale per (row, 128-wide K block)
    B   uint8 [G, N, K]      e4m3 bytes; B[g, n, k] is element (k, n) of the paper's B^g
    SB  float [G, ceil(N/128), ceil(K/128)]   one scale per 128x128 block of B^g
    group_offsets int [G+1]  rows of group g are [off[g], off[g+1])
    rows  optional 1-D array of global row indices; only those rows are
          evaluated (each one by the same formula), in the order given.

    Returns a dict:
      "rows"  int64 [R]      global row index of each output row
      "group" int64 [R]      the group each row belongs to
      "D"     float64 [R, N] the block-scaled dot products
      "C"     uint16 [R, N]  bfloat16 (out="bf16") or binary16 (out="f16") bit patterns of D, one RNE rounding
      "S"     float64 [R, N] (with_abs_sum) sum_kb |sa*sb| * sum_k |a*b| -- the
              magnitude against which a float32 accumulation error is bounded
    Scales are dequantisation multipliers: real value = dec(byte) * scale.
    """
    A = np.asarray(A)
    B = np.asarray(B)
    off = np.asarray(group_offsets, dtype=np.int64)
    K = A.shape[1]
    N = B.shape[1]
    SA = np.asarray(SA, dtype=np.float64)
    SB = np.asarray(SB, dtype=np.float64)
    G, KB, NB = _check_shapes(A, SA, B, SB, off, N, K)
    assert np.all(np.diff(off) >= 0) and off[0] >= 0 and off[-1] <= A.shape[0]

    if rows is None:
        rows = np.arange(off[0], off[-1], dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    assert np.all((rows >= off[0]) & (rows < off[-1])), "row outside every group"
    # group of row r: the g with off[g] <= r < off[g+1] (empty groups are skipped by 'right')
    grp = np.searchsorted(off, rows, side="right") - 1

    R = rows.shape[0]
    D = np.zeros((R, N), dtype=np.float64)
    S = np.zeros((R, N), dtype=np.float64) if with_abs_sum else None
    col_block = np.arange(N) // SCALE_BLOCK            # n -> index of its 128-wide N block

    for g in np.unique(grp):
        sel = np.nonzero(grp == g)[0]
        rg = rows[sel]
        Dg = np.zeros((sel.shape[0], N), dtype=np.float64)
        Sg = np.zeros_like(Dg) if with_abs_sum else None
        for kb in range(KB):
            k0, k1 = kb * SCALE_BLOCK, min((kb + 1) * SCALE_BLOCK, K)
            a = e4m3_decode(A[rg, k0:k1])               # [R_g, <=128] float64
            b = e4m3_decode(B[g, :, k0:k1])             # [N,   <=128] float64
            inner = a @ b.T                             # exact (see module docstring)
            scale = SA[rg, kb][:, None] * SB[g, col_block, kb][None, :]   # exact product
            Dg += scale * inner                         # the only rounding steps: * and +=
            if with_abs_sum:
                Sg += np.abs(scale) * (np.abs(a) @ np.abs(b).T)
        D[sel] = Dg
        if with_abs_sum:
            S[sel] = Sg

    assert out in ("bf16", "f16")
    out = {"rows": rows, "group": grp, "D": D, "C": bf16_bits_from_f64(D) if out == "bf16" else f16_bits_from_f64(D)}
    if with_abs_sum:
        out["S"] = S
    return out


# ----------------------------------------------------------------------------
# the variable-K grouped GEMM of training (the weight gradient of the same expert
# layer).  The paper's title names training next to inference and its Sec. 4
# points at the kernels around the grouped GEMM, but it defines neither layouts
# nor scale granularity for this one: the definition below is this build's own
# reading, and the function is PARITY UNPINNED AGAINST THE PAPER (its pins in
# tests/test_oracle_pins.py are exact rationals, closed forms and the reduction
# of its one-group case to grouped_gemm above).
# ----------------------------------------------------------------------------
def grouped_gemm_wgrad(XT, SX, DYT, SDY, group_offsets, with_abs_sum=False, out="fp32"):
    """dW^g = dY^g^T X^g for every group, the contraction running over the group's rows (tokens).

    XT   uint8 [K, M_total]   e4m3 bytes of X transposed: XT[k, r] is feature k of token r
    SX   float [ceil(M_total/128), K]   one scale per (block of 128 tokens, feature), the scales of one block
         contiguous; the token blocks are [128 j, 128 j + 128) of the concatenated token axis, whatever the groups
         are (a block may hold tokens of two or more groups)
    DYT  uint8 [N, M_total]   e4m3 bytes of dY transposed
    SDY  float [ceil(M_total/128), N]
    group_offsets int [G+1]   tokens of group g are [off[g], off[g+1])

        dW[g, n, k] = sum_{j ascending} ( SDY[j, n] * SX[j, k] )
                                        * ( sum_{r in block j and in group g} dec(DYT[n, r]) * dec(XT[k, r]) )

    Tokens outside the group contribute nothing, whatever their bytes are (NaN codes included).  A group without
    tokens gives zeros.  Returns {"D": float64 [G, N, K], "W": float32 [G, N, K] (D rounded once, to nearest even),
    "S": float64 [G, N, K] (with_abs_sum): sum_j |sdy*sx| * sum_r |dy*x|}; with out="bf16" also "C": the bfloat16
    bits of D rounded once, to nearest even (the two-byte output of the library's option).
    The inner sums are exact in float64 (at most 128 products, each a multiple of 2^-18 below 2^18) and so is
    sdy*sx; only the accumulation over j rounds, in ascending order.
    """
    XT = np.asarray(XT)
    DYT = np.asarray(DYT)
    off = np.asarray(group_offsets, dtype=np.int64)
    assert XT.dtype == np.uint8 and DYT.dtype == np.uint8 and XT.ndim == 2 and DYT.ndim == 2
    K, M_total = XT.shape
    N = DYT.shape[0]
    assert DYT.shape[1] == M_total
    MB = -(-M_total // SCALE_BLOCK)
    SX = np.asarray(SX, dtype=np.float64)
    SDY = np.asarray(SDY, dtype=np.float64)
    assert SX.shape == (MB, K) and SDY.shape == (MB, N)
    G = off.shape[0] - 1
    assert np.all(np.diff(off) >= 0) and off[0] >= 0 and off[-1] <= M_total
    D = np.zeros((G, N, K), dtype=np.float64)
    S = np.zeros((G, N, K), dtype=np.float64) if with_abs_sum else None
    for g in range(G):
        lo, hi = int(off[g]), int(off[g + 1])
        if hi <= lo:
            continue
        for j in range(lo // SCALE_BLOCK, -(-hi // SCALE_BLOCK)):
            r0, r1 = max(j * SCALE_BLOCK, lo), min((j + 1) * SCALE_BLOCK, hi)
            dy = e4m3_decode(DYT[:, r0:r1])             # [N, <=128]
            x = e4m3_decode(XT[:, r0:r1])               # [K, <=128]
            inner = dy @ x.T                            # exact
            scale = SDY[j][:, None] * SX[j][None, :]
            D[g] += scale * inner
            if with_abs_sum:
                S[g] += np.abs(scale) * (np.abs(dy) @ np.abs(x).T)
    with np.errstate(over="ignore", invalid="ignore"):
        res = {"D": D, "W": D.astype(np.float32)}       # float64 -> float32 is one RNE step
    if with_abs_sum:
        res["S"] = S
    assert out in ("fp32", "bf16")
    if out == "bf16":
        res["C"] = bf16_bits_from_f64(D)
    return res


# ----------------------------------------------------------------------------
# the padded formulation the paper compares against (Sec. 3: padding of A and
# S_A to multiples of 128 rows per group, then the same GEMM, then removal of
# the pad rows)
# ----------------------------------------------------------------------------
def padded_offsets(group_offsets, align=SCALE_BLOCK):
    """Offsets of the groups after each is rounded up to a multiple of `align` rows."""
    off = np.asarray(group_offsets, dtype=np.int64)
    sizes = np.diff(off)
    padded = -(-sizes // align) * align
    return np.concatenate([[0], np.cumsum(padded)]).astype(np.int64)


def pad(A, SA, group_offsets, align=SCALE_BLOCK, rows_cap=None):
    """Copy every group to its aligned offset; pad rows of A and SA are zero.

    Returns (A_pad uint8 [M_pad, K], SA_pad [M_pad, KB], padded_offsets [G+1]).
    `rows_cap` >= M_pad allocates a larger (zero) tail, as a caller that cannot
    know M_pad in advance would.
    """
    A = np.asarray(A)
    SA = np.asarray(SA)
    off = np.asarray(group_offsets, dtype=np.int64)
    poff = padded_offsets(off, align)
    M_pad = int(poff[-1]) if rows_cap is None else int(rows_cap)
    assert M_pad >= poff[-1]
    A_pad = np.zeros((M_pad, A.shape[1]), dtype=A.dtype)    # byte 0x00 decodes to +0
    SA_pad = np.zeros((M_pad, SA.shape[1]), dtype=SA.dtype)
    for g in range(off.shape[0] - 1):
        n = off[g + 1] - off[g]
        A_pad[poff[g]:poff[g] + n] = A[off[g]:off[g + 1]]
        SA_pad[poff[g]:poff[g] + n] = SA[off[g]:off[g + 1]]
    return A_pad, SA_pad, poff


def unpad(C_pad, group_offsets, padded_off, M_total, fill=0):
    """Gather the valid rows of a padded output back to the concatenated layout."""
    off = np.asarray(group_offsets, dtype=np.int64)
    poff = np.asarray(padded_off, dtype=np.int64)
    C = np.full((M_total, C_pad.shape[1]), fill, dtype=C_pad.dtype)
    for g in range(off.shape[0] - 1):
        n = off[g + 1] - off[g]
        C[off[g]:off[g + 1]] = C_pad[poff[g]:poff[g] + n]
    return C


# ----------------------------------------------------------------------------
# the paper's own residual-row store rule (Sec. 2.2, Eq. 1-2 and App. B).  The
# HIP path does not use it (bounded stores replace it); it is kept so that the
# claim "exactly the residual rows are written, none beyond" can be checked
# for the paper's mechanism as well as for ours.
# ----------------------------------------------------------------------------
def descriptor_pool(block_M):
    """Row counts of the store shapes of Eq. 1: 2^i for 0 <= i <= floor(log2 block_M)."""
    return [1 << i for i in range(int(block_M).bit_length())]


def two_phase_cover(M_g, block_M=128):
    """Row ranges (inclusive) of the two stores that write the residual block of a group.

    res = M_g mod block_M; p = 2^floor(log2 res) is the selected shape (Eq. 2).
    Phase 1 copies tile rows [0, p-1] to group rows [M_g-res, M_g-res+p-1];
    phase 2 copies tile rows [res-p, res-1] to group rows [M_g-p, M_g-1].
    Returns None when res == 0 (no residual block; log2(0) is undefined in Eq. 2).
    """
    res = M_g % block_M
    if res == 0:
        return None
    p = 1 << (res.bit_length() - 1)
    return {
        "res": res,
        "rows_desc": p,
        "phase1_tile": (0, p - 1),
        "phase1_group": (M_g - res, M_g - res + p - 1),
        "phase2_tile": (res - p, res - 1),
        "phase2_group": (M_g - p, M_g - 1),
    }


# ----------------------------------------------------------------------------
# the step before the GEMM: rows -> e4m3 bytes + 1x128 scales, group-contiguous
# ----------------------------------------------------------------------------
E4M3_MAX = 448.0


def e4m3_encode_rne(y: np.ndarray) -> np.ndarray:
    """uint8 codes of float32 values with |y| <= 448 (or NaN): round to nearest e4m3 value, ties to the even code.

    Written from the format's definition (the one e4m3_decode_table spells out), not from a bit trick:
    below 2^-6 the representable values are m * 2^-9 (m = 0..8, 8 being the smallest normal), from there on
    (1 + m/8) * 2^e.  Every intermediate below is exact in float64.  NaN -> 0x7F (sign dropped).
    """
    y = np.asarray(y, dtype=np.float32)
    a = np.abs(y.astype(np.float64))
    nan = np.isnan(a)
    a = np.where(nan, 0.0, a)
    assert np.all(a <= E4M3_MAX), "values must be clamped to the e4m3 range first"
    code = np.zeros(a.shape, dtype=np.int64)
    sub = a < 2.0 ** -6
    code[sub] = np.rint(a[sub] * 2.0 ** 9).astype(np.int64)          # 0..8; 8 is the code of 2^-6
    nrm = ~sub
    m, e = np.frexp(a[nrm])                                         # a = m * 2^e, m in [0.5, 1)
    e = e - 1                                                       # a = (2m) * 2^e, 2m in [1, 2)
    steps = np.rint((2.0 * m - 1.0) * 8.0).astype(np.int64)         # 0..8; 8 carries into the exponent
    code[nrm] = ((e + 7) << 3) + steps                              # the carry is the integer addition
    code = np.where(nan, 0x7F, code)
    sign = np.where(np.signbit(y) & ~nan, 0x80, 0)
    return (code | sign).astype(np.uint8)


AMAX_FLOOR = 2.0 ** -100     # blocks whose largest magnitude is below this are quantised as if it were this


def quantize_rows(X_bf16_bits: np.ndarray, row_src=None, M_total=None):
    """Producer of the GEMM's A operand (the kernel the padding-free layout lets run on valid rows only,
    Sec. 4): output row r is input row row_src[r] (identity if None), cut into 1x128 blocks along K
    (Sec. 2.1: 1x128 scaling of A).  The paper does not define the quantiser; the recipe fixed here is the
    usual one, per block and in float32 as the hardware does it:

        amax  = max( max |x| over the block with NaNs skipped, 2^-100 )
        scale = amax / 448                                    (a dequantisation multiplier)
        inv   = 448 / amax
        byte  = e4m3_encode_rne( clamp(x * inv, -448, 448) ), NaN stays NaN (0x7F)

    (an infinite amax gives scale = inf, inv = 0: finite elements become 0, infinite ones NaN.)
    A source index outside [0, T) stands for a row of zeros (zero bytes, scales 2^-100 / 448).
    Returns (uint8 [M_total, K], float32 [M_total, K/128]).
    """
    Xb = np.asarray(X_bf16_bits)
    assert Xb.dtype == np.uint16 and Xb.ndim == 2
    T, K = Xb.shape
    assert K % SCALE_BLOCK == 0
    KB = K // SCALE_BLOCK
    if row_src is None:
        row_src = np.arange(T if M_total is None else M_total, dtype=np.int64)
    row_src = np.asarray(row_src, dtype=np.int64)
    M = row_src.shape[0]
    A = np.zeros((M, K), dtype=np.uint8)
    SA = np.full((M, KB), np.float32(AMAX_FLOOR) / np.float32(E4M3_MAX), dtype=np.float32)
    ok = (row_src >= 0) & (row_src < T)
    x = (Xb[row_src[ok]].astype(np.uint32) << 16).view(np.float32).reshape(-1, KB, SCALE_BLOCK)
    with np.errstate(invalid="ignore", divide="ignore", over="ignore"):
        amax = np.nan_to_num(np.abs(x), nan=0.0, posinf=np.inf).max(axis=2).astype(np.float32)
        amax = np.maximum(amax, np.float32(AMAX_FLOOR))
        scale = (amax / np.float32(E4M3_MAX)).astype(np.float32)     # float32 divisions, correctly rounded
        inv = (np.float32(E4M3_MAX) / amax).astype(np.float32)
        y = (x * inv[:, :, None]).astype(np.float32)                 # one float32 rounding per element
        y = np.where(np.isnan(y), y, np.clip(y, -E4M3_MAX, E4M3_MAX)).astype(np.float32)
    A[ok] = e4m3_encode_rne(y).reshape(-1, K)
    SA[ok] = scale
    return A, SA


def quantize_cols(X_bf16_bits: np.ndarray, row_src=None, M_total=None):
    """Producer of the operands of grouped_gemm_wgrad: the quantiser of quantize_rows applied ALONG THE TOKENS.
    Token r of the output is input row row_src[r] (identity if None); feature k of it goes to XT[k][r], and the
    1x128 blocks of Sec. 2.1 run along r: block j of feature k holds tokens [128 j, 128 j + 128) of the output order
    (whatever the groups are), the last block those that exist.  Per block the recipe of quantize_rows, in float32:

        amax  = max( max |x| over the block's tokens with NaNs skipped, 2^-100 )
        scale = amax / 448,  inv = 448 / amax,  byte = e4m3_encode_rne( clamp(x * inv, -448, 448) ), NaN -> 0x7F

    A source index outside [0, T) stands for a row of zeros.  The paper defines neither this operation nor its
    layouts (PARITY UNPINNED AGAINST THE PAPER, like grouped_gemm_wgrad); it is pinned to quantize_rows, which is
    the same recipe on the transposed matrix.
    Returns (uint8 [K, M_total], float32 [ceil(M_total / 128), K]).
    """
    Xb = np.asarray(X_bf16_bits)
    assert Xb.dtype == np.uint16 and Xb.ndim == 2
    T, K = Xb.shape
    if row_src is None:
        row_src = np.arange(T if M_total is None else M_total, dtype=np.int64)
    row_src = np.asarray(row_src, dtype=np.int64)
    M = row_src.shape[0]
    MB = -(-M // SCALE_BLOCK)
    ok = (row_src >= 0) & (row_src < T)
    x = np.zeros((M, K), dtype=np.float32)
    x[ok] = (Xb[row_src[ok]].astype(np.uint32) << 16).view(np.float32)
    XT = np.zeros((K, M), dtype=np.uint8)
    SX = np.empty((MB, K), dtype=np.float32)
    for j in range(MB):
        blk = x[j * SCALE_BLOCK:(j + 1) * SCALE_BLOCK]               # [tokens of the block, K]
        with np.errstate(invalid="ignore", divide="ignore", over="ignore"):
            amax = np.nan_to_num(np.abs(blk), nan=0.0, posinf=np.inf).max(axis=0).astype(np.float32)
            amax = np.maximum(amax, np.float32(AMAX_FLOOR))
            SX[j] = (amax / np.float32(E4M3_MAX)).astype(np.float32)
            inv = (np.float32(E4M3_MAX) / amax).astype(np.float32)
            y = (blk * inv[None, :]).astype(np.float32)
            y = np.where(np.isnan(y), y, np.clip(y, -E4M3_MAX, E4M3_MAX)).astype(np.float32)
        XT[:, j * SCALE_BLOCK:j * SCALE_BLOCK + blk.shape[0]] = e4m3_encode_rne(y).T
    return XT, SX


def swiglu_rows(H_bf16_bits: np.ndarray) -> np.ndarray:
    """The activation between the two grouped GEMMs of an expert MLP, on group-contiguous rows: H [M, 2I] is the
    output of the first GEMM (columns [0, I): gate projection, [I, 2I): up projection),

        act[r, j] = bf16_round_to_nearest_even( silu(H[r, j]) * H[r, I + j] ),   silu(g) = g / (1 + exp(-g))

    evaluated in float64 and rounded once.  Returns bf16 bits [M, I].  (Not in the paper; it is one of the
    neighbouring kernels that Sec. 4 says run unchanged on the padding-free layout.)
    """
    Hb = np.asarray(H_bf16_bits)
    assert Hb.dtype == np.uint16 and Hb.ndim == 2 and Hb.shape[1] % 2 == 0
    half = Hb.shape[1] // 2
    g = f64_from_bf16_bits(Hb[:, :half])
    u = f64_from_bf16_bits(Hb[:, half:])
    with np.errstate(over="ignore", invalid="ignore"):
        act = g / (1.0 + np.exp(-g)) * u
    return bf16_bits_from_f64(act)


def swiglu_quantize_rows(H_bf16_bits: np.ndarray):
    """swiglu_rows followed by quantize_rows on its bf16 result: (act bits, A, SA)."""
    act = swiglu_rows(H_bf16_bits)
    A, SA = quantize_rows(act)
    return act, A, SA
