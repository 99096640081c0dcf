"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Every test here needs a real MI355X.  Inputs are seeded and synthetic; the tolerance is defined and
justified in tests/gg_testlib.py.
"""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc
from workloads import CONFIGS, WorkloadConfig, group_sizes, make_problem

from gg_testlib import ParityAccumulator, assert_parity, bits_of, np_problem, raw_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CANARY = 0x7B7B          # bf16 bit pattern that no test result produces in bulk


# variants of the second kernel that also come in the instantiation for partial tiles, a short last K block and an odd
# number of K blocks
RB_ANY_SHAPE = {"256x256/1x8w/3s-rb", "192x256/1x8w/3s-rb", "224x256/1x8w/3s-rb", "128x256/1x8w/3s-rb"}


def variants_for(N, K):
    """Tile variants that take this shape (K a multiple of 128): N a multiple of the tile width; the second kernel
    ("-rb") fetches three K blocks ahead (K > 256) and alternates two register sets by K-block parity, so only its
    any-shape instantiations take an odd number of K blocks."""
    out = []
    for v in range(gg.num_variants()):
        name = gg.variant_name(v)
        bn = int(name.split("/")[0].split("x")[1])
        rb_ok = "-rb" not in name or (K > 256 and (K % 256 == 0 or name in RB_ANY_SHAPE))
        if N % bn == 0 and rb_ok and not ("-k2" in name and K % 256 != 0):
            out.append(v)
    return out


def family_of(v):
    """Variants whose results agree bit for bit: the arithmetic per element does not depend on the tiling.  "-rbk"
    variants feed the 128 products of a scale block to the matrix instruction in another order, and "-k2" (split-K)
    variants add the two halves of the K loop as two partial sums, so each of these is a family of its own."""
    name = gg.variant_name(v) if v >= 0 else ""
    return "k-permuted" if name.endswith("-rbk") else "split-k" if name.endswith("-k2") else "plain"


def canary_C(M, N):
    return torch.full((M, N), CANARY, dtype=torch.int16, device=DEV).view(torch.bfloat16)


def run_gpu(dev, M, N, variant=-1, C=None):
    A, SA, B, SB, off = dev
    if C is None:
        C = canary_C(M, N)
    gg.grouped_gemm(A, SA, B, SB, off, C=C, variant=variant)
    torch.cuda.synchronize()
    return bits_of(C)


# ----------------------------------------------------------------------------------------------
def test_library_loaded_is_the_in_tree_hip_build():
    lib = gg.load_library()
    assert lib.gg_fp8_version() >= 100
    assert gg.library_path().endswith("paper_2508_16584_amd/libgg_fp8.so")
    assert gg.num_variants() >= 1


def test_tiny_config_every_variant_full_compare():
    p = make_problem(CONFIGS["tiny"])
    host = np_problem(p)
    ref = orc.grouped_gemm(*host, with_abs_sum=True)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    first = {}
    for v in [-1] + variants_for(p["N"], p["K"]):
        got = run_gpu(dev, p["M_total"], p["N"], v)
        assert_parity(got, ref, what=f"tiny variant {v}")
        # The arithmetic per element does not depend on the tiling: all variants of one kernel agree bit for
        # bit.  Variants named "-rbk" feed the 128 products of a scale block to the matrix instruction in
        # another order, so they form a family of their own.
        family = family_of(v)
        if family not in first:
            first[family] = got
        assert np.array_equal(got, first[family]), f"variant {v} differs from the first of its family"


@pytest.mark.parametrize("sizes,N,K", [
    ([1], 256, 128),
    ([0, 0, 0], 256, 256),
    ([127, 128, 129], 256, 384),
    ([253], 128, 256),                       # the group of the paper's worked example (App. B)
    ([381, 0, 125], 128, 256),               # and of its figure caption
    ([16, 17, 15, 1, 0, 31, 33], 512, 512),
    ([255, 256, 257, 0, 1], 256, 256),
    ([700], 384, 640),                       # N a multiple of 128 but not of 256
    ([40, 0, 3, 130], 2304, 4096),           # row pitch 4096: the K loop of a tile starts at a block that depends on its column
])
def test_edge_group_sizes_every_variant(sizes, N, K):
    cfg = WorkloadConfig("edge", 50, len(sizes), K, N, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    host = np_problem(p)
    ref = orc.grouped_gemm(*host, with_abs_sum=True)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    for v in [-1] + variants_for(N, K):
        got = run_gpu(dev, p["M_total"], N, v)
        assert_parity(got, ref, empirical=p["M_total"] * N >= 50000, what=f"sizes {sizes} variant {v}")


def test_many_empty_groups_and_a_wide_output():
    rng = np.random.default_rng(61)
    # 1000 groups of which 988 are empty: the tile walk steps over long runs of zero-row groups
    sizes = np.zeros(1000, dtype=np.int64)
    sizes[rng.choice(1000, size=12, replace=False)] = rng.integers(1, 70, size=12)
    cfg = WorkloadConfig("empties", 53, 1000, 512, 256, 0, "custom", "latency")
    p = make_problem(cfg, sizes=sizes)
    ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    for v in (-1, 0, 5, 14):
        assert_parity(run_gpu(dev, p["M_total"], 256, v), ref, empirical=False, what=f"1000 groups variant {v}")
    # N = 16384: 64 column tiles per row tile, walked in chunks of 8
    cfg = WorkloadConfig("wide", 54, 2, 512, 16384, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array([37, 200]))
    ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    for v in (-1, 1, 2, 12):
        assert_parity(run_gpu(dev, p["M_total"], 16384, v), ref, what=f"N=16384 variant {v}")


def test_operands_written_by_a_kernel_just_before_the_launch():
    """Short groups take the instantiation whose weight fetches carry the streaming cache policy, and C is stored with
    it: operands that a device kernel on the same stream wrote immediately before the launch (still in the caches, over
    memory that held other bytes) must be what the GEMM reads, and a device kernel right behind it must read the C it
    wrote.  Several rounds with new contents in the same buffers."""
    rng = np.random.default_rng(62)
    cfg = WorkloadConfig("fresh", 55, 24, 1024, 512, 0, "custom", "latency")
    sizes = rng.integers(0, 120, 24)
    bufs = None
    for rnd in range(3):
        p = make_problem(cfg, sizes=sizes, seed=550 + rnd)
        ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
        src = {k: p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets")}
        if bufs is None:
            bufs = {k: torch.empty_like(v) for k, v in src.items()}
            C = torch.empty((p["M_total"], 512), dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        for k in bufs:
            bufs[k].copy_(src[k])                       # device kernels; no synchronisation before the GEMM
        for v in (-1, 0, 3):
            gg.grouped_gemm(bufs["A"], bufs["SA"], bufs["B"], bufs["SB"], bufs["group_offsets"], C=C, variant=v)
            C2 = C.clone()                              # a device kernel reading C right behind the GEMM
            torch.cuda.synchronize()
            assert_parity(bits_of(C2), ref, empirical=False, what=f"round {rnd} variant {v}")


@pytest.mark.timeout(600)
def test_largest_k_and_largest_n_the_library_takes():
    """K = 2^22 and N = 2^21, the limits of the argument check (32-bit offsets inside a tile).  The oracle evaluates
    the columns of one 128-column block at a time (16 columns of each of two blocks), every row."""
    def references(A, SA, B, SB, off, blocks):
        refs = []
        for blk in blocks:
            cols = np.arange(blk * 128, blk * 128 + 8)
            cols = np.concatenate([cols, cols + 120])
            refs.append((blk, cols, orc.grouped_gemm(A, SA, np.ascontiguousarray(B[:, cols, :]), SB[:, blk:blk + 1, :], off,
                                                     with_abs_sum=True)))
        return refs

    def check_columns(refs, got, what):
        for blk, cols, ref in refs:
            assert_parity(got[:, cols], ref, empirical=False, what=f"{what}, column block {blk}")

    rng = np.random.default_rng(71)
    # ---- K = 2^22: 32768 K blocks, 4 MB per row
    sizes, N, K = [3, 0, 14], 256, 1 << 22
    G, M, KB = len(sizes), sum(sizes), K // 128
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    A = rng.integers(0x20, 0x48, (M, K), dtype=np.uint8) | (rng.integers(0, 2, (M, K), dtype=np.uint8) << 7)
    B = rng.integers(0x20, 0x48, (G, N, K), dtype=np.uint8) | (rng.integers(0, 2, (G, N, K), dtype=np.uint8) << 7)
    SA = rng.uniform(0.5, 2.0, (M, KB)).astype(np.float32)
    SB = rng.uniform(0.5, 2.0, (G, N // 128, KB)).astype(np.float32)
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    refs = references(A, SA, B, SB, off, (0, 1))
    first = None
    for v in [-1] + [u for u in range(gg.num_variants()) if gg.variant_name(u) in ("160x256/2x4w/3s", "256x256/1x8w/3s-rb", "128x256/2x4w/3s-k2")]:
        got = run_gpu(dev, M, N, v)
        if family_of(v) == "plain":
            first = got if first is None else first
            assert np.array_equal(got, first), f"K = 2^22: variant {v} differs"
        check_columns(refs, got, f"K = 2^22 variant {v}")
    del dev, A, B, refs
    # ---- N = 2^21: 8192 column tiles of 256, 16384 scale blocks
    sizes, N, K = [5, 2], 1 << 21, 128
    G, M = len(sizes), sum(sizes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    A = rng.integers(0, 0x7F, (M, K), dtype=np.uint8)
    B = rng.integers(0x28, 0x40, (G, N, K), dtype=np.uint8) | (rng.integers(0, 2, (G, N, K), dtype=np.uint8) << 7)
    SA = rng.uniform(0.5, 2.0, (M, 1)).astype(np.float32)
    SB = rng.uniform(0.5, 2.0, (G, N // 128, 1)).astype(np.float32)
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    refs = references(A, SA, B, SB, off, (0, 1, 8191, 16382, 16383))
    for v in (-1, 2, 3):
        C = canary_C(M + 2, N)
        gg.grouped_gemm(*dev, C=C[1:M + 1], variant=v)
        torch.cuda.synchronize()
        bits = bits_of(C)
        assert (bits[0] == CANARY).all() and (bits[M + 1] == CANARY).all()
        check_columns(refs, bits[1:M + 1], f"N = 2^21 variant {v}")
        assert (bits[1:M + 1] != CANARY).any(axis=0).all(), "a column was never written"


@pytest.mark.parametrize("K", [512, 768, 1024, 1536])
def test_several_tiles_per_workgroup_every_element(K):
    """More tiles than workgroups at a size the oracle can check in full: every workgroup walks through several
    tiles, which is where both kernels hand their fetch pipeline from one tile to the next (the first kernel's last
    K blocks fetch for the next tile; the second kernel's K loop runs on into it).  K = 512 is the shortest K loop
    the second kernel takes (4 K blocks: the hand-over starts in the first K step); the others have a main loop too,
    of one, two and four turns."""
    sizes, N = [700, 0, 1300, 37, 1800, 191], 4096
    cfg = WorkloadConfig("walk", 55, len(sizes), K, N, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    first = {}
    for v in [-1] + variants_for(N, K):
        bm = 128 if v < 0 else int(gg.variant_name(v).split("x")[0])
        if v >= 0 and (sum(-(-m // bm) for m in sizes) * (N // 256) <= 256 or bm < 128):
            continue                                   # fewer tiles than workgroups, or a tile for short groups
        got = run_gpu(dev, p["M_total"], N, v)
        assert_parity(got, ref, what=f"K={K} variant {v}")
        family = family_of(v)
        first.setdefault(family, got)
        assert np.array_equal(got, first[family]), f"variant {v} differs from the first of its family"


def test_rows_outside_the_groups_and_guard_bands_are_untouched():
    # groups cover rows [5, 5+sum) of a larger buffer; C has guard rows before and after
    rng = np.random.default_rng(60)
    sizes, N, K = [130, 0, 67], 256, 512
    host, dev = raw_problem(rng, sizes, N, K, DEV)
    A, SA, B, SB, off = host
    pre, post = 5, 9
    M = A.shape[0] + pre + post
    A2 = np.concatenate([rng.integers(0, 120, (pre, K), dtype=np.uint8), A, rng.integers(0, 120, (post, K), dtype=np.uint8)])
    SA2 = np.concatenate([np.ones((pre, K // 128), np.float32), SA, np.ones((post, K // 128), np.float32)])
    off2 = (off + pre).astype(np.int32)
    ref = orc.grouped_gemm(A2, SA2, B, SB, off2, with_abs_sum=True)
    dev2 = tuple(torch.from_numpy(x).to(DEV) for x in (A2, SA2, B, SB, off2))
    for v in variants_for(N, K):
        guard = 64
        buf = torch.full(((M + 2 * guard), N), CANARY, dtype=torch.int16, device=DEV)
        C = buf[guard:guard + M].view(torch.bfloat16)
        got = run_gpu(dev2, M, N, v, C=C)
        allb = buf.cpu().numpy().view(np.uint16)
        assert np.all(allb[:guard + pre] == CANARY), f"variant {v} wrote before the first group"
        assert np.all(allb[guard + pre + A.shape[0]:] == CANARY), f"variant {v} wrote past the last group"
        assert_parity(got[pre:pre + A.shape[0]], ref, empirical=False, what=f"guard variant {v}")


def test_raw_bytes_full_dynamic_range_hard_bound():
    # every e4m3 code (subnormals included), arbitrary scales: only the hard bound applies
    rng = np.random.default_rng(61)
    sizes, N, K = [77, 200, 3], 256, 512
    host, dev = raw_problem(rng, sizes, N, K, DEV)
    ref = orc.grouped_gemm(*host, with_abs_sum=True)
    for v in variants_for(N, K):
        got = run_gpu(dev, int(sum(sizes)), N, v)
        assert_parity(got, ref, empirical=False, what=f"raw bytes variant {v}")


def test_closed_forms_are_exact():
    # (a) all ones: every output is K * alpha * beta exactly
    N, K, M = 256, 640, 70
    A = torch.full((M, K), 0x38, dtype=torch.uint8, device=DEV)
    B = torch.full((2, N, K), 0x38, dtype=torch.uint8, device=DEV)
    SA = torch.full((M, K // 128), 0.375, device=DEV)
    SB = torch.full((2, N // 128, K // 128), 1.25, device=DEV)
    off = torch.tensor([0, 33, 70], dtype=torch.int32, device=DEV)
    got = bits_of(gg.grouped_gemm(A, SA, B, SB, off))
    want = orc.bf16_bits_from_f64(np.array([K * 0.375 * 1.25]))[0]
    assert np.all(got == want)
    # (b) small integers and power-of-two scales: every intermediate is exact in fp32, so the GPU must
    #     reproduce the oracle bit for bit, not merely within tolerance
    rng = np.random.default_rng(62)
    small = [0x00, 0x38, 0x40, 0x44, 0xB8, 0xC0, 0xC4]        # 0, 1, 2, 3, -1, -2, -3
    host, dev = raw_problem(rng, [129, 1, 62], 256, 512, DEV, byte_choices=small, scale_pow2=True)
    ref = orc.grouped_gemm(*host)
    for v in variants_for(256, 512):
        got = run_gpu(dev, 192, 256, v)
        assert np.array_equal(got, ref["C"]), f"variant {v}"
    # (c) subnormal codes only on the A side, B = +-1: products are exact multiples of 2^-9
    sub = [0x01, 0x02, 0x03, 0x04, 0x05, 0x06, 0x07, 0x81, 0x83, 0x87]
    host, dev = raw_problem(rng, [40, 90], 256, 256, DEV, byte_choices=sub, scale_pow2=True)
    Bh = np.where(rng.integers(0, 2, host[2].shape) == 1, 0x38, 0xB8).astype(np.uint8)
    host = (host[0], host[1], Bh, host[3], host[4])
    dev = (dev[0], dev[1], torch.from_numpy(Bh).to(DEV), dev[3], dev[4])
    ref = orc.grouped_gemm(*host)
    got = run_gpu(dev, 130, 256)
    assert np.array_equal(got, ref["C"])


def test_mfma_truncation_model_matches_the_tolerance_derivation():
    """The tolerance in gg_testlib.py rests on how the gfx950 FP8 MFMA adds its 128 products: in groups of 8
    consecutive k, each product truncated toward zero to a grid 2^-13 below the group's largest product.
    Drive exactly that case through the library: k0 = 256*256, k1..7 = 15*1, k8 = -256*256.  Exact: 105.
    Under the model the first group gives 2^16 + 7*8, the second -2^16: 56.  Still inside the hard bound."""
    M, N, K = 16, 256, 128
    A = np.zeros((M, K), np.uint8)
    B = np.zeros((1, N, K), np.uint8)
    A[:, 0], A[:, 1:8], A[:, 8] = 0x78, 0x57, 0xF8          # 256, 15, -256
    B[0, :, 0], B[0, :, 1:8], B[0, :, 8] = 0x78, 0x38, 0x78  # 256, 1, 256
    SA = np.ones((M, 1), np.float32)
    SB = np.ones((1, 2, 1), np.float32)
    off = np.array([0, M], np.int32)
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    assert np.all(ref["D"] == 105.0)
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    got = run_gpu(dev, M, N)
    assert_parity(got, ref, empirical=False, what="mfma truncation case")
    assert np.all(orc.f64_from_bf16_bits(got) == 56.0), "the MFMA no longer truncates as measured: re-derive the tolerance"


@pytest.mark.parametrize("ea", [-6, -2, 2, 6, 8])
@pytest.mark.parametrize("eb", [-6, 0, 8])
def test_mfma_truncation_model_over_a_range_of_magnitudes(ea, eb):
    """The same construction swept over magnitudes: one product 2^(ea+eb) at k = 0, seven products v * 1 behind it in
    the same group of 8 (v another e4m3 value in every row), -2^(ea+eb) in the next group.  Exact result 7 v; the
    model of gg_testlib.mfma_block_model says 7 * trunc(v) on the grid 2^-13 below the group's largest product.  The
    GPU must give the model's value bit for bit, for large products that swallow v entirely, for products below v
    (v sets the grid and nothing is lost), and everything between: the floor of the tolerance then rests on a model
    that is checked, not on one case."""
    from gg_testlib import mfma_block_model
    dec = orc.e4m3_decode_table()
    pow2_code = lambda e: np.uint8((e + 7) << 3)             # e4m3 code of 2^e, -6 <= e <= 8
    v_codes = np.array([0x01, 0x07, 0x0F, 0x15, 0x1B, 0x22, 0x2D, 0x33, 0x39, 0x3F, 0x46, 0x4D, 0x57, 0x5E, 0x66, 0x6F], np.uint8)
    M, N, K = 16, 256, 128
    A = np.zeros((M, K), np.uint8)
    B = np.zeros((1, N, K), np.uint8)
    A[:, 0], A[:, 8] = pow2_code(ea), pow2_code(ea) | 0x80
    A[:, 1:8] = v_codes[:, None]
    B[0, :, 0], B[0, :, 8] = pow2_code(eb), pow2_code(eb)
    B[0, :, 1:8] = 0x38                                       # 1.0
    SA = np.ones((M, 1), np.float32)
    SB = np.ones((1, 2, 1), np.float32)
    off = np.array([0, M], np.int32)
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    assert np.array_equal(ref["D"][:, 0], 7.0 * dec[v_codes])
    model = mfma_block_model(dec[A][:, None, :], dec[B[0]][None, :, :])          # [M, N]
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    got = run_gpu(dev, M, N)
    assert_parity(got, ref, empirical=False, what=f"mfma truncation sweep 2^{ea} * 2^{eb}")
    assert np.array_equal(got, orc.bf16_bits_from_f64(model)), (
        f"2^{ea} * 2^{eb}: GPU {orc.f64_from_bf16_bits(got)[:, 0]} against the model's {model[:, 0]} (exact {ref['D'][:, 0]})")


def test_group_permutation_permutes_row_blocks_bitwise():
    cfg = WorkloadConfig("perm", 51, 4, 512, 256, 0, "custom", "latency")
    sizes = np.array([150, 0, 31, 260])
    p = make_problem(cfg, sizes=sizes)
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    base = run_gpu(dev, p["M_total"], 256)
    perm = [3, 1, 0, 2]
    off = p["group_offsets"].numpy()
    rows = np.concatenate([np.arange(off[g], off[g + 1]) for g in perm])
    A_p, SA_p = p["A"][rows], p["SA"][rows]
    off_p = np.concatenate([[0], np.cumsum(sizes[perm])]).astype(np.int32)
    dev_p = (A_p.to(DEV), SA_p.to(DEV), p["B"][perm].to(DEV), p["SB"][perm].to(DEV), torch.from_numpy(off_p).to(DEV))
    got = run_gpu(dev_p, p["M_total"], 256)
    assert np.array_equal(got, base[rows])


def test_nan_stays_in_its_row_and_column():
    rng = np.random.default_rng(63)
    host, dev = raw_problem(rng, [20, 30], 256, 256, DEV)
    A, SA, B, SB, off = host
    A[7, 200] = 0x7F
    B[1, 100, 3] = 0xFF
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    got = run_gpu(dev, 50, 256)
    assert_parity(got, ref, empirical=False, what="nan")     # checks the NaN pattern too


def test_untrusted_offsets_never_write_outside_C():
    # decreasing and out-of-range offsets: results are unspecified, but nothing outside C[0:M] is written
    rng = np.random.default_rng(64)
    host, dev = raw_problem(rng, [100, 100, 100], 256, 512, DEV)
    M = 300
    bad = torch.tensor([-5, 250, 120, 100000], dtype=torch.int32, device=DEV)
    assert gg.check_offsets(bad, M) == 6          # GG_ERR_OFFSETS
    assert gg.check_offsets(dev[4], M) == 0
    for v in variants_for(256, 512):
        guard = 300
        buf = torch.full(((M + 2 * guard), 256), CANARY, dtype=torch.int16, device=DEV)
        C = buf[guard:guard + M].view(torch.bfloat16)
        gg.grouped_gemm(dev[0], dev[1], dev[2], dev[3], bad, C=C, variant=v)
        torch.cuda.synchronize()
        allb = buf.cpu().numpy().view(np.uint16)
        assert np.all(allb[:guard] == CANARY) and np.all(allb[guard + M:] == CANARY)


# ---------------------------------------------------------------------------------------------- pad path
@pytest.mark.parametrize("sizes,N,K", [
    ([130, 0, 1, 128, 253, 127], 256, 256),
    ([5, 300, 64], 256, 512),
    ([3, 140, 64], 2304, 4096),              # rotated K loops: same order in both paths
])
def test_pad_path_equals_padding_free_path_bitwise(sizes, N, K):
    cfg = WorkloadConfig("pad", 52, len(sizes), K, N, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    A_h, SA_h, B_h, SB_h, off_h = np_problem(p)
    A, SA, B, SB, off = (p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    M = p["M_total"]
    cap = gg.padded_rows_cap(len(sizes), M)
    assert cap == 128 * (-(-M // 128) + len(sizes))
    A_pad, SA_pad, poff = gg.pad(A, SA, off)
    torch.cuda.synchronize()
    # pad kernel against the oracle's pad (bytes, scales and offsets exactly) on the rows of the padded problem
    A_ref, SA_ref, poff_ref = orc.pad(A_h, SA_h, off_h)
    m_pad = int(poff_ref[-1])
    assert np.array_equal(poff.cpu().numpy(), poff_ref.astype(np.int32))
    assert np.array_equal(A_pad.cpu().numpy()[:m_pad], A_ref)
    assert np.array_equal(SA_pad.cpu().numpy()[:m_pad], SA_ref)
    # rows between the padded problem's end and the capacity belong to no group and keep what the caller put there,
    # in both storage orders of the scales
    K = A.shape[1]
    for km in (False, True):
        A_can = torch.full((cap, K), 0xA5, dtype=torch.uint8, device=DEV)
        SA_can = torch.full((K // 128, cap) if km else (cap, K // 128), -7.0, dtype=torch.float32, device=DEV)
        gg.pad(A, SA.t().contiguous() if km else SA, off, cap, sa_kmajor=km, A_pad=A_can, SA_pad=SA_can)
        torch.cuda.synchronize()
        sa_rows = SA_can.t() if km else SA_can
        assert np.array_equal(A_can.cpu().numpy()[:m_pad], A_ref) and np.array_equal(sa_rows.cpu().numpy()[:m_pad], SA_ref)
        assert m_pad < cap and (A_can[m_pad:] == 0xA5).all() and (sa_rows[m_pad:] == -7.0).all()
    # padded GEMM + unpad against the padding-free GEMM: bitwise equal on valid rows (Sec. 3.2)
    C_pad = gg.grouped_gemm_padded(A_pad, SA_pad, B, SB, poff)
    C2 = gg.unpad(C_pad, off, poff, M)
    C1 = gg.grouped_gemm(A, SA, B, SB, off)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(C1), bits_of(C2))
    # pad rows inside the padded groups are zeros (zero A rows, zero scales)
    cp = bits_of(C_pad)
    valid = np.zeros(cap, bool)
    for g in range(len(sizes)):
        valid[poff_ref[g]:poff_ref[g] + sizes[g]] = True
    inside = np.arange(cap) < poff_ref[-1]
    assert not (cp[inside & ~valid] & 0x7FFF).any()
    # and the oracle agrees with both
    ref = orc.grouped_gemm(A_h, SA_h, B_h, SB_h, off_h, with_abs_sum=True)
    assert_parity(bits_of(C1), ref, what="pad-free")


# ---------------------------------------------------------------------------------------------- full sizes
def sampled_rows(off, rng, every=97, max_groups=None):
    """First row, last two rows of (a subset of) the groups plus every `every`-th row."""
    G = len(off) - 1
    groups = np.arange(G)
    if max_groups is not None and G > max_groups:
        groups = np.sort(rng.choice(G, size=max_groups, replace=False))
    rows = []
    for g in groups:
        n = off[g + 1] - off[g]
        if n > 0:
            rows += [off[g], off[g + 1] - 1, max(off[g], off[g + 1] - 2)]
            rows += list(range(off[g], off[g + 1], every))
    return np.unique(np.array(rows, dtype=np.int64))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["gate_up", "down", "decode", "many_small"])
def test_full_size_configs_every_element(name):
    """The four full-size workloads in the launch configurations bench.py times (automatic variant; the plain call
    with row-major activation scales, which is the headline, and the K-block-major order through the _ex call):
    EVERY row and column of both outputs against the oracle, group by group, plus "no row outside the groups is
    written, every row inside is" by canaries."""
    cfg = CONFIGS[name]
    p = make_problem(cfg, device=DEV)
    off = p["group_offsets"].cpu().numpy()
    assert np.array_equal(np.diff(off), group_sizes(cfg))
    M, N = p["M_total"], cfg.N
    C_row = canary_C(M, N)
    gg.grouped_gemm(p["A"], p["SA"], p["B"], p["SB"], p["group_offsets"], C=C_row)                    # gg_fp8_grouped_gemm
    C_km = canary_C(M, N)
    gg.grouped_gemm(p["A"], p["SA"].t().contiguous(), p["B"], p["SB"], p["group_offsets"], C=C_km, sa_kmajor=True)
    torch.cuda.synchronize()
    acc_row, acc_km = ParityAccumulator(f"{name}, row-major scales"), ParityAccumulator(f"{name}, K-block-major scales")
    for g in range(cfg.G):
        r0, r1 = int(off[g]), int(off[g + 1])
        if r1 == r0:
            continue
        ref = orc.grouped_gemm(p["A"][r0:r1].cpu().numpy(), p["SA"][r0:r1].cpu().numpy(), p["B"][g:g + 1].cpu().numpy(),
                               p["SB"][g:g + 1].cpu().numpy(), np.array([0, r1 - r0]), with_abs_sum=True)
        acc_row.add(bits_of(C_row[r0:r1]), ref)
        acc_km.add(bits_of(C_km[r0:r1]), ref)
    s_row, s_km = acc_row.finish(), acc_km.finish()
    assert s_row["elements"] == M * N == s_km["elements"]
    print(f"\n{name}: all {M} rows x {N} columns, row-major {s_row}, K-block-major {s_km}")
    # the two storage orders of the scales give the same bits
    assert torch.equal(C_row.view(torch.int16), C_km.view(torch.int16))


@pytest.mark.parametrize("N,K,G,M", [
    (3072, 8192, 4, 8192),
    (8192, 3072, 32, 8192),
    (5120, 6144, 16, 16384),
    (7168, 4096, 32, 65536),
])
def test_paper_grid_points_with_the_papers_size_generator(N, K, G, M):
    """Points of the paper's sweep grid (Sec. 3.1) with group sizes from its generator (App. C.1): sampled rows
    against the oracle, every row written, and pad + GEMM + unpad equal to the padding-free result bit for bit."""
    from workloads.configs import paper_group_sizes
    rng = np.random.default_rng([20250816, N, K, G, M])
    sizes = paper_group_sizes(M, G, rng)
    assert sizes.sum() == M and (sizes >= 0).all()
    cfg = WorkloadConfig("grid", 70, G, K, N, M, "custom", "mfma")
    p = make_problem(cfg, device=DEV, sizes=sizes)
    off = p["group_offsets"].cpu().numpy()
    C = canary_C(M, N)
    gg.grouped_gemm(p["A"], p["SA"], p["B"], p["SB"], p["group_offsets"], C=C)
    torch.cuda.synchronize()
    rows = sampled_rows(off, rng, every=211)
    grp = np.searchsorted(off, rows, side="right") - 1
    used = np.unique(grp)
    ridx = torch.from_numpy(rows).to(DEV)
    A_s, SA_s = p["A"][ridx].cpu().numpy(), p["SA"][ridx].cpu().numpy()
    B_s = p["B"][torch.from_numpy(used).to(DEV)].cpu().numpy()
    SB_s = p["SB"][torch.from_numpy(used).to(DEV)].cpu().numpy()
    off_s = np.concatenate([[0], np.cumsum([(grp == g).sum() for g in used])])
    ref = orc.grouped_gemm(A_s, SA_s, B_s, SB_s, off_s, with_abs_sum=True)
    stats = assert_parity(bits_of(C[ridx]), ref, what=f"grid N={N} K={K} G={G} M={M}")
    print(f"\ngrid N={N} K={K} G={G} M={M}: sizes {sizes.min()}..{sizes.max()}, {len(rows)} rows: {stats}")
    assert (C.view(torch.int16) != CANARY).any(dim=1).all()
    # the comparison path of the sweep
    cap = gg.padded_rows_cap(G, M)
    A_pad, SA_pad, poff = gg.pad(p["A"], p["SA"], p["group_offsets"], cap)
    C_pad = torch.zeros((cap, N), dtype=torch.bfloat16, device=DEV)
    gg.grouped_gemm_padded(A_pad, SA_pad, p["B"], p["SB"], poff, C_pad)
    C2 = canary_C(M, N)
    gg.unpad(C_pad, p["group_offsets"], poff, M, C=C2)
    torch.cuda.synchronize()
    assert int(poff[-1].item()) == int(np.sum(128 * ((sizes + 127) // 128)))
    assert torch.equal(C.view(torch.int16), C2.view(torch.int16))
    # the same two paths with the activation scales stored K-block-major (what the sweep times by default)
    SAk = p["SA"].t().contiguous()
    C3 = canary_C(M, N)
    gg.grouped_gemm(p["A"], SAk, p["B"], p["SB"], p["group_offsets"], C=C3, sa_kmajor=True)
    A_pad, SA_pad, poff = gg.pad(p["A"], SAk, p["group_offsets"], cap, sa_kmajor=True)
    gg.grouped_gemm_padded(A_pad, SA_pad, p["B"], p["SB"], poff, C_pad, sa_kmajor=True)
    C4 = canary_C(M, N)
    gg.unpad(C_pad, p["group_offsets"], poff, M, C=C4)
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), C3.view(torch.int16)) and torch.equal(C.view(torch.int16), C4.view(torch.int16))


# ---------------------------------------------------------------------------------------------- binary16 output
def f16_bits_of(C: torch.Tensor) -> np.ndarray:
    return C.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def test_binary16_output_every_variant():
    p = make_problem(CONFIGS["tiny"])
    host = np_problem(p)
    ref = orc.grouped_gemm(*host, with_abs_sum=True, out="f16")
    dev = tuple(p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    first = {}
    for v in [-1] + variants_for(p["N"], p["K"]):
        C = torch.full((p["M_total"], p["N"]), 0x7B7B, dtype=torch.int16, device=DEV).view(torch.float16)
        gg.grouped_gemm(*dev, C=C, variant=v)
        torch.cuda.synchronize()
        got = f16_bits_of(C)
        assert_parity(got, ref, what=f"binary16 variant {v}", fmt="f16")
        family = family_of(v)
        first.setdefault(family, got)
        assert np.array_equal(got, first[family])


def test_binary16_output_ragged_groups_overflow_and_untouched_rows():
    rng = np.random.default_rng(71)
    sizes, N, K = [130, 0, 67, 1], 256, 384
    host, dev = raw_problem(rng, sizes, N, K, DEV)
    A, SA, B, SB, off = host
    # raw bytes with scales up to 4 x 4: many results leave binary16's range (|x| >= 65520 -> infinity)
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True, out="f16")
    assert np.isinf(orc.f64_from_f16_bits(ref["C"])).mean() > 0.01
    M = int(off[-1])
    C = torch.full((M + 4, N), 0x7B7B, dtype=torch.int16, device=DEV).view(torch.float16)
    gg.grouped_gemm(*dev, C=C[:M])
    torch.cuda.synchronize()
    bits = f16_bits_of(C)
    assert (bits[M:] == 0x7B7B).all()
    assert_parity(bits[:M], ref, empirical=False, what="binary16 raw bytes", fmt="f16")


def test_binary16_output_full_size_sampled_rows():
    p = make_problem(CONFIGS["gate_up"], device=DEV)
    C = gg.grouped_gemm(p["A"], p["SA"], p["B"], p["SB"], p["group_offsets"], out_dtype=torch.float16)
    torch.cuda.synchronize()
    off = p["group_offsets"].cpu().numpy()
    rows = sampled_rows(off, np.random.default_rng(72), every=211)
    ridx = torch.from_numpy(rows).to(DEV)
    ref = orc.grouped_gemm(p["A"][ridx].cpu().numpy(), p["SA"][ridx].cpu().numpy(), p["B"].cpu().numpy(),
                           p["SB"].cpu().numpy(), np.concatenate([[0], np.cumsum(np.bincount(
                               np.searchsorted(off, rows, side="right") - 1, minlength=p["G"]))]),
                           with_abs_sum=True, out="f16")
    assert_parity(f16_bits_of(C[ridx]), ref, what="binary16 gate_up", fmt="f16")


# ---------------------------------------------------------------------------------------------- ragged N and K
@pytest.mark.parametrize("sizes,N,K", [
    ([70, 0, 129, 5], 200, 208),             # one partial tile, one short K block after a full one
    ([33, 260], 136, 144),                   # 8 columns and 16 bytes past the first block
    ([300], 392, 528),                       # 256 + 136 columns: full tile then partial; 4 K blocks + 16 bytes
    ([17, 1, 140], 8, 16),                   # the smallest legal shape
    ([64, 64], 648, 4112),                   # K = 4096 + 16
    ([50, 3], 1032, 128),                    # N ragged only
    ([50, 3], 256, 1008),                    # K ragged only
    ([300, 17, 0, 513], 264, 272),           # 3 K blocks, the last 16 bytes long; second tile 8 columns wide
    ([100, 260, 31], 512, 640),              # whole blocks, an odd number of them
    ([30, 500], 776, 912),                   # 8 K blocks with a short last one; N = 3 * 256 + 8
])
def test_ragged_n_and_k_every_variant_that_takes_them(sizes, N, K):
    """Ceilings in Table 1 of the paper: the last scale block along K and along N may be short.  The library takes
    any N % 8 == 0 and K % 16 == 0 (16-byte stores and fetches); raw bytes and uniform scales, hard bound."""
    rng = np.random.default_rng(900 + N + K)
    sizes = np.asarray(sizes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    M, G = int(off[-1]), len(sizes)
    KB, NB = -(-K // 128), -(-N // 128)
    A = rng.integers(0, 256, (M, K), dtype=np.uint8)
    B = rng.integers(0, 256, (G, N, K), dtype=np.uint8)
    A[(A & 0x7F) == 0x7F] = 0x35
    B[(B & 0x7F) == 0x7F] = 0x35
    A[(A & 0x78) > 0x58] &= 0xBF             # keep magnitudes moderate: no overflow of bf16 with scales up to 4
    SA = rng.uniform(0.25, 4.0, (M, KB)).astype(np.float32)
    SB = rng.uniform(0.25, 4.0, (G, NB, KB)).astype(np.float32)
    ref = orc.grouped_gemm(A, SA, B, SB, off, with_abs_sum=True)
    dev = tuple(torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    first, supported = None, []
    for v in [-1] + list(range(gg.num_variants())):
        C = torch.full((M + 3, N), CANARY, dtype=torch.int16, device=DEV).view(torch.bfloat16)
        try:
            gg.grouped_gemm(*dev, C=C[:M], variant=v)
        except gg.GGError as e:                 # a variant built for whole tiles and whole K blocks only says so
            assert e.status == 3 and v >= 0
            continue
        supported.append(v)
        torch.cuda.synchronize()
        bits = bits_of(C)
        assert (bits[M:] == CANARY).all(), f"variant {v} wrote past the last row"
        assert_parity(bits[:M], ref, empirical=False, what=f"N={N} K={K} variant {v}")
        first = bits if first is None else first
        assert np.array_equal(bits, first), f"variant {v} differs from the others"          # (no split-K variant takes these shapes)
    # the automatic choice and the tiles it draws from always work; the second kernel needs three K blocks
    names = {gg.variant_name(v) for v in supported if v >= 0}
    assert -1 in supported and {"160x256/2x4w/3s", "128x128/2x4w/4s", "128x256/2x4w/3s", "32x256/1x8w/4s"} <= names
    rb = {n for n in names if "-rb" in n}
    assert rb == (RB_ANY_SHAPE if K > 256 else set())


def test_ragged_shapes_pad_path_bitwise_and_exact_case():
    rng = np.random.default_rng(77)
    sizes, N, K = [130, 0, 1, 67], 200, 336
    host, dev = None, None
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    M, G = int(off[-1]), len(sizes)
    KB, NB = -(-K // 128), -(-N // 128)
    # small integers and power-of-two scales: every intermediate is exact, the GPU must equal the oracle bit for bit
    ints = np.array([0x00, 0x38, 0xB8, 0x40, 0xC0, 0x44], dtype=np.uint8)       # 0, 1, -1, 2, -2, 3
    A = ints[rng.integers(0, len(ints), (M, K))]
    B = ints[rng.integers(0, len(ints), (G, N, K))]
    SA = (2.0 ** rng.integers(-2, 3, (M, KB))).astype(np.float32)
    SB = (2.0 ** rng.integers(-2, 3, (G, NB, KB))).astype(np.float32)
    ref = orc.grouped_gemm(A, SA, B, SB, off)
    At, SAt, Bt, SBt, offt = (torch.from_numpy(x).to(DEV) for x in (A, SA, B, SB, off))
    C1 = gg.grouped_gemm(At, SAt, Bt, SBt, offt)
    A_pad, SA_pad, poff = gg.pad(At, SAt, offt)
    C_pad = gg.grouped_gemm_padded(A_pad, SA_pad, Bt, SBt, poff)
    C2 = gg.unpad(C_pad, offt, poff, M)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(C1), ref["C"])
    assert np.array_equal(bits_of(C2), ref["C"])
