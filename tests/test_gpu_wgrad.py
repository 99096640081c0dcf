"""GPU parity of gg_fp8_grouped_gemm_wgrad (the variable-K grouped GEMM of training) against oracle.grouped_gemm_wgrad,
element by element, through the C ABI.

Tolerance, from the kernel's arithmetic (the same derivation as for the forward GEMM, see gg_testlib): one FP8 matrix
instruction per 128-token block (products truncated inside groups of 8: at most 7 * 2^-13 of the block's absolute
sum), the factor sx * sdy rounded to fp32, fp32 accumulation over J blocks, fp32 output:
    |gpu - D| <= ulp_fp32(D) + 2^-10 * S          (HARD, every element)
and on quantised normal data (EMPIRICAL, regression guard; observed: 2^-15.7 * S -- an fp32 result shows the
truncation that the forward GEMM's bfloat16 rounding hides)
    |gpu - D| <= ulp_fp32(D) + 2^-13 * S.
Where every intermediate is exact (small integers, power-of-two scales) the GPU must equal the oracle bit for bit.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def random_bytes(rng, shape):
    b = rng.integers(0, 256, size=shape, dtype=np.uint8)
    b[(b & 0x7F) == 0x7F] = 0x3A
    return b


def quantised_normal(rng, rows, M_total, std=1.0):
    """e4m3 bytes [rows, M_total] and scales [ceil(M_total/128), rows] of normal samples, by torch's float8 cast
    (test input only)."""
    MB = -(-M_total // 128)
    x = torch.from_numpy(rng.standard_normal((rows, MB * 128)).astype(np.float32) * std)
    amax = x.view(rows, MB, 128).abs().amax(dim=2).clamp_min(1e-30)
    scale = amax / 448.0
    q = (x.view(rows, MB, 128) / scale[:, :, None]).clamp(-448, 448).to(torch.float8_e4m3fn)
    return q.view(torch.uint8).view(rows, MB * 128)[:, :M_total].contiguous().numpy(), scale.t().contiguous().numpy()


def run_gpu(XT, SX, DYT, SDY, off):
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(DEV)
    dW = gg.grouped_gemm_wgrad(t(XT, torch.uint8), t(SX, torch.float32), t(DYT, torch.uint8), t(SDY, torch.float32),
                               t(np.asarray(off), torch.int32))
    torch.cuda.synchronize()
    return dW.cpu().numpy()


def assert_wgrad_parity(got, ref, floor, what):
    D, S = ref["D"], ref["S"]
    assert got.shape == D.shape and got.dtype == np.float32
    nan = np.isnan(D)
    assert np.array_equal(np.isnan(got), nan), f"{what}: NaN pattern differs"
    ok = ~nan
    err = np.abs(np.where(ok, got.astype(np.float64) - D, 0.0))
    ulp = np.spacing(np.abs(np.where(ok, D, 1.0)).astype(np.float32)).astype(np.float64)
    bound = ulp + floor * np.where(ok, S, 0.0)
    bad = np.argwhere(err > bound)
    assert bad.size == 0, f"{what}: {bad.shape[0]} elements outside the bound, first {bad[:3].tolist()}: got {got[tuple(bad[0])]} want {D[tuple(bad[0])]}"
    return float(np.mean(got[ok] == ref["W"][ok])), float(np.max(err / np.maximum(np.where(ok, S, 0.0), 1e-300)))


def test_wgrad_groups_that_cut_through_token_blocks_full_range_bytes():
    rng = np.random.default_rng(31)
    M_total, N, K = 304, 128, 256
    off = [0, 37, 37, 130, 291, 300, 304]
    XT, DYT = random_bytes(rng, (K, M_total)), random_bytes(rng, (N, M_total))
    SX = rng.uniform(0.25, 4.0, (3, K)).astype(np.float32)
    SDY = rng.uniform(0.25, 4.0, (3, N)).astype(np.float32)
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    got = run_gpu(XT, SX, DYT, SDY, off)
    assert_wgrad_parity(got, ref, 2.0 ** -10, "edge groups")
    assert np.all(got[1] == 0)                                             # the empty group is written, as zeros


def test_wgrad_several_tiles_quantised_data_and_unowned_tokens():
    rng = np.random.default_rng(32)
    M_total, N, K = 2000, 384, 768                                          # 3 x 3 output tiles per group
    off = [16, 16, 555, 1403, 1404, 1990]                                   # tokens [0,16) and [1990,2000) belong to nobody
    XT, SX = quantised_normal(rng, K, M_total)
    DYT, SDY = quantised_normal(rng, N, M_total, std=0.02)
    XT[:, :16] = 0x7F                                                       # NaN codes outside every group
    DYT[:, 1990:] = 0xFF
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    assert not np.isnan(ref["D"]).any()
    got = run_gpu(XT, SX, DYT, SDY, off)
    equal, worst = assert_wgrad_parity(got, ref, 2.0 ** -13, "quantised")
    assert np.all(got[0] == 0)


def test_wgrad_blocked_tile_list_every_element():
    """4 k tiles x 8 n tiles: the tile list runs in blocks of 4 x 8 (the order the full-size layers take); every
    element of every group against the oracle, with a group that ends on a block boundary, one inside a single block
    and an empty one."""
    rng = np.random.default_rng(36)
    M_total, N, K = 912, 1024, 1024
    off = [5, 5, 256, 300, 901]                                             # [5,5) empty, [5,256) ends on a boundary, [256,300) inside one block
    XT, SX = quantised_normal(rng, K, M_total)
    DYT, SDY = quantised_normal(rng, N, M_total, std=0.02)
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    got = run_gpu(XT, SX, DYT, SDY, off)
    assert_wgrad_parity(got, ref, 2.0 ** -13, "blocked tile list")
    assert np.all(got[0] == 0)
    # the same problem with exact inputs: bit-equal, so a tile written to the wrong place cannot hide in the tolerance
    codes = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0], np.uint8)
    XTe, DYTe = codes[rng.integers(0, 6, (K, M_total))], codes[rng.integers(0, 6, (N, M_total))]
    SXe = (2.0 ** rng.integers(-3, 4, SX.shape)).astype(np.float32)
    SDYe = (2.0 ** rng.integers(-3, 4, SDY.shape)).astype(np.float32)
    assert np.array_equal(run_gpu(XTe, SXe, DYTe, SDYe, off), orc.grouped_gemm_wgrad(XTe, SXe, DYTe, SDYe, off)["W"])


@pytest.mark.parametrize("seed", range(12))
def test_wgrad_seeded_random_shapes(seed):
    """Random group counts, sizes (many groups empty or shorter than a block, so that tiles which only store zeros
    and tiles of one masked block follow each other), unowned tokens at both ends, N and K from one tile to a blocked
    tile list; every element against the oracle, and bit-equal on exact inputs."""
    rng = np.random.default_rng(4000 + seed)
    N = int(rng.choice([128, 256, 384, 1024]))
    K = int(rng.choice([256, 512, 1024]))
    G = int(rng.integers(1, 9))
    sizes = rng.integers(0, 400, G) * (rng.random(G) < 0.7)
    sizes[rng.integers(0, G)] = int(rng.integers(1, 40))
    lead = int(rng.integers(0, 3)) * 7
    total = lead + int(sizes.sum()) + int(rng.integers(0, 30))
    M_total = max(16, -(-total // 16) * 16)
    off = (lead + np.concatenate([[0], np.cumsum(sizes)])).astype(np.int64)
    XT, SX = quantised_normal(rng, K, M_total)
    DYT, SDY = quantised_normal(rng, N, M_total, std=0.02)
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    got = run_gpu(XT, SX, DYT, SDY, off)
    assert_wgrad_parity(got, ref, 2.0 ** -13, f"seed {seed}: G={G} N={N} K={K} M={M_total} sizes={sizes.tolist()}")
    codes = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0], np.uint8)
    XTe, DYTe = codes[rng.integers(0, 6, (K, M_total))], codes[rng.integers(0, 6, (N, M_total))]
    SXe = (2.0 ** rng.integers(-3, 4, SX.shape)).astype(np.float32)
    SDYe = (2.0 ** rng.integers(-3, 4, SDY.shape)).astype(np.float32)
    assert np.array_equal(run_gpu(XTe, SXe, DYTe, SDYe, off), orc.grouped_gemm_wgrad(XTe, SXe, DYTe, SDYe, off)["W"])


def run_gpu_bf16(XT, SX, DYT, SDY, off):
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(DEV)
    dW = gg.grouped_gemm_wgrad(t(XT, torch.uint8), t(SX, torch.float32), t(DYT, torch.uint8), t(SDY, torch.float32),
                               t(np.asarray(off), torch.int32), out_bf16=True)
    torch.cuda.synchronize()
    return dW.view(torch.int16).cpu().numpy().view(np.uint16)


def test_wgrad_bfloat16_output():
    """gg_fp8_grouped_gemm_wgrad_ex with GG_OUT_BF16: the same sums rounded once to bfloat16; the bounds of the
    forward GEMM's bfloat16 output (gg_testlib.assert_parity: hard max(ulp, ulp/2 + 2^-10 S) on every element,
    empirical ulp/2 + 2^-15 S and the shares within one ulp and bit-equal on quantised data), bit-equal on exact
    inputs, zeros for a group without tokens."""
    from gg_testlib import assert_parity
    rng = np.random.default_rng(37)
    M_total, N, K = 1200, 384, 1024
    off = [16, 16, 555, 1100, 1190]
    XT, SX = quantised_normal(rng, K, M_total)
    DYT, SDY = quantised_normal(rng, N, M_total, std=0.02)
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True, out="bf16")
    got = run_gpu_bf16(XT, SX, DYT, SDY, off)
    assert_parity(got, ref, empirical=True, what="bf16 weight gradient")
    assert np.all(got[0] == 0)
    codes = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0], np.uint8)
    XTe, DYTe = codes[rng.integers(0, 6, (K, M_total))], codes[rng.integers(0, 6, (N, M_total))]
    SXe = (2.0 ** rng.integers(-3, 4, SX.shape)).astype(np.float32)
    SDYe = (2.0 ** rng.integers(-3, 4, SDY.shape)).astype(np.float32)
    ref_e = orc.grouped_gemm_wgrad(XTe, SXe, DYTe, SDYe, off, out="bf16")
    assert np.array_equal(run_gpu_bf16(XTe, SXe, DYTe, SDYe, off), ref_e["C"])
    # full-range bytes (hard bound only) and a NaN inside a group
    XTr, DYTr = random_bytes(rng, (K, M_total)), random_bytes(rng, (N, M_total))
    XTr[5, 700] = 0x7F
    ref_r = orc.grouped_gemm_wgrad(XTr, SX, DYTr, SDY, off, with_abs_sum=True, out="bf16")
    ref_r["S"] = np.nan_to_num(ref_r["S"], nan=0.0)
    assert_parity(run_gpu_bf16(XTr, SX, DYTr, SDY, off), ref_r, empirical=False, what="bf16 weight gradient, raw bytes")


def test_wgrad_exact_where_every_intermediate_is_exact():
    rng = np.random.default_rng(33)
    M_total, N, K = 1024 + 48, 128, 256
    off = [0, 5, 133, 700, 1072]
    codes = np.array([0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0], np.uint8)        # 0, 1, 2, 3, -1, -2
    XT, DYT = codes[rng.integers(0, 6, (K, M_total))], codes[rng.integers(0, 6, (N, M_total))]
    MB = -(-M_total // 128)
    SX = (2.0 ** rng.integers(-3, 4, (MB, K))).astype(np.float32)
    SDY = (2.0 ** rng.integers(-3, 4, (MB, N))).astype(np.float32)
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off)
    got = run_gpu(XT, SX, DYT, SDY, off)
    assert np.array_equal(got, ref["W"])


def test_wgrad_nan_inside_a_group_reaches_its_feature_row_in_that_group_only():
    rng = np.random.default_rng(34)
    M_total, N, K = 512, 128, 256
    off = [0, 200, 512]
    XT, DYT = random_bytes(rng, (K, M_total)), random_bytes(rng, (N, M_total))
    SX = np.ones((4, K), np.float32)
    SDY = np.ones((4, N), np.float32)
    XT[77, 300] = 0x7F
    ref = orc.grouped_gemm_wgrad(XT, SX, DYT, SDY, off, with_abs_sum=True)
    ref["S"] = np.nan_to_num(ref["S"], nan=0.0)
    got = run_gpu(XT, SX, DYT, SDY, off)
    assert_wgrad_parity(got, ref, 2.0 ** -10, "nan")
    assert np.isnan(got).sum() == N and np.all(np.isnan(got[1, :, 77]))


def test_wgrad_no_tokens_at_all_writes_zeros():
    off = torch.zeros(4, dtype=torch.int32, device=DEV)
    dW = torch.full((3, 128, 256), 7.0, dtype=torch.float32, device=DEV)
    e8 = torch.empty((256, 0), dtype=torch.uint8, device=DEV)
    gg.grouped_gemm_wgrad(e8, torch.empty((0, 256), dtype=torch.float32, device=DEV), e8[:128],
                          torch.empty((0, 128), dtype=torch.float32, device=DEV), off, dW=dW)
    torch.cuda.synchronize()
    assert torch.count_nonzero(dW).item() == 0


def test_wgrad_full_size_sampled_rows_of_both_operands():
    """gate_up's layer in training: 8 experts, 8192 tokens, hidden 7168, 4096 rows of dY^T.  The GPU computes all of
    dW [8, 4096, 7168]; the oracle the 96 x 160 sampled (row of dY^T, feature) pairs of every group (rows of the two
    operands are independent, so the oracle runs on the sampled rows alone)."""
    from workloads import CONFIGS, group_sizes
    cfg = CONFIGS["gate_up"]
    sizes = group_sizes(cfg)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    M_total, N, K = int(off[-1]), cfg.N, cfg.K
    rng = np.random.default_rng(35)
    XT, SX = quantised_normal(rng, K, M_total)
    DYT, SDY = quantised_normal(rng, N, M_total, std=0.02)
    got = run_gpu(XT, SX, DYT, SDY, off)
    n_sel = np.sort(rng.choice(N, 96, replace=False))
    k_sel = np.sort(rng.choice(K, 160, replace=False))
    n_sel[0], n_sel[-1], k_sel[0], k_sel[-1] = 0, N - 1, 0, K - 1        # the corners of the output are among them
    ref = orc.grouped_gemm_wgrad(XT[k_sel], SX[:, k_sel], DYT[n_sel], SDY[:, n_sel], off, with_abs_sum=True)
    sub = got[:, n_sel][:, :, k_sel]
    assert_wgrad_parity(sub, ref, 2.0 ** -13, "full size")
    assert np.isfinite(got).all()
