"""GPU test of gg_fp8_grouped_gemm_splitk_noalloc, the entry point for callers that cannot allocate: through the C
ABI, against gg_fp8_grouped_gemm_ex with the same split-K variant and a caller's workspace (bit for bit) and against
the oracle, on two calls in a row, the second with a smaller input; sizes beyond the built-in scratch are refused."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from oracle import gg_oracle as orc
from workloads import WorkloadConfig, make_problem

from gg_testlib import assert_parity, bits_of, np_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CANARY = 0x7B7B


def split_k_variant():
    return next(v for v in range(gg.num_variants()) if gg.variant_name(v) == "128x256/2x4w/3s-k2")


def run_both(sizes, N, K, seed):
    cfg = WorkloadConfig("noalloc", seed, len(sizes), K, N, 0, "custom", "latency")
    p = make_problem(cfg, sizes=np.array(sizes))
    ref = orc.grouped_gemm(*np_problem(p), with_abs_sum=True)
    A, SA, B, SB, off = (p[k].to(DEV) for k in ("A", "SA", "B", "SB", "group_offsets"))
    G, M = len(sizes), p["M_total"]
    v = split_k_variant()
    lib = gg.load_library()
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the existing entry point: split-K variant, the caller's workspace
    need = gg.workspace_bytes(G, M, N, K, v)
    assert need == 2 * M * N * 4
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    C_ws = torch.full((M, N), CANARY, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    rc = lib.gg_fp8_grouped_gemm_ex(vp(A), vp(SA), vp(B), vp(SB), vp(off), vp(C_ws), G, M, N, K, vp(ws), need, stream, v, 0)
    assert rc == 0, gg.status_str(rc)
    # the new one: no workspace argument at all
    C_na = torch.full((M, N), CANARY, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    rc = lib.gg_fp8_grouped_gemm_splitk_noalloc(vp(A), vp(SA), vp(B), vp(SB), vp(off), vp(C_na), G, M, N, K, stream, v, 0)
    assert rc == 0, gg.status_str(rc)
    torch.cuda.synchronize()
    got_ws, got_na = bits_of(C_ws), bits_of(C_na)
    assert np.array_equal(got_ws, got_na), "the built-in scratch changed the result"
    assert_parity(got_na, ref, empirical=M * N >= 50000, what=f"no-alloc split-K, sizes {sizes}")
    return got_na


def test_noalloc_entry_point_twice_second_call_smaller():
    run_both([300, 0, 77, 129, 1], 512, 1024, 81)          # 507 rows x 512: several tiles and a ragged tail
    run_both([40, 3, 0, 130], 256, 512, 82)                # a smaller problem on the same scratch, right after
    # beyond the built-in scratch: refused before anything is enqueued
    lib = gg.load_library()
    p = ctypes.c_void_p(0x1000)
    cap = gg.noalloc_max_elements()
    assert cap == 4 << 20
    assert lib.gg_fp8_grouped_gemm_splitk_noalloc(p, p, p, p, p, p, 2, cap // 256 + 1, 256, 512, None, -1, 0) == 4   # GG_ERR_WORKSPACE
    assert lib.gg_fp8_grouped_gemm_splitk_noalloc(p, p, p, p, p, p, 2, 100, 256, 512, None, 0, 0) == 3               # not a split-K variant
    assert lib.gg_fp8_grouped_gemm_splitk_noalloc(p, p, p, p, p, p, 2, 100, 256, 384, None, -1, 0) == 3              # odd number of K blocks
