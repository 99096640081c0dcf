"""Host-side checks of the C-ABI library: it loads, exports what include/gg_fp8.h declares, and
rejects bad arguments before anything is enqueued.  No GPU is needed: every call below returns
from argument validation."""
import ctypes
import os
import re

import pytest

import paper_2508_16584_amd as gg
from paper_2508_16584_amd import binding

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "gg_fp8.h")

GG_OK, GG_ERR_NULL, GG_ERR_SHAPE, GG_ERR_UNSUPPORTED, GG_ERR_WORKSPACE, GG_ERR_HIP, GG_ERR_OFFSETS = range(7)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gg.library_path()):
        gg.build_library()
    return gg.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gg_fp8_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in gg_fp8.h but not exported"
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_probe_library_exports_what_its_header_declares():
    """include/gg_probe.h: the measurement probes live in a library of their own (no compute call without a GPU)."""
    header = os.path.join(os.path.dirname(HEADER), "gg_probe.h")
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(gg_probe_\w+)\s*\(", text)))
    assert names == ["gg_probe_gemm_kstep", "gg_probe_hbm", "gg_probe_issue_mix", "gg_probe_lds_fetch", "gg_probe_mfma",
                     "gg_probe_wgrad_parts"]
    if not os.path.exists(gg.probe_library_path()):
        gg.build_library()
    probe = gg.load_probe_library()
    for n in names:
        assert hasattr(probe, n), f"{n} is declared in gg_probe.h but not exported"
    # argument checks come before any GPU call
    out = ctypes.c_double(0.0)
    assert probe.gg_probe_mfma(4, 0, 10, ctypes.byref(out)) != 0 and probe.gg_probe_mfma(0, 0, 0, ctypes.byref(out)) != 0
    assert probe.gg_probe_issue_mix(1, 1, 1, 10, ctypes.byref(out)) != 0 and probe.gg_probe_issue_mix(0, 0, 0, 0, ctypes.byref(out)) != 0
    assert probe.gg_probe_hbm(2, 4096, 1, ctypes.byref(out)) != 0 and probe.gg_probe_hbm(0, 100, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_lds_fetch(3, 3, 1, ctypes.byref(out), ctypes.byref(out)) != 0
    assert probe.gg_probe_lds_fetch(0, 8, 1, ctypes.byref(out), ctypes.byref(out)) != 0
    # tile height, build, shape (n % 256, k % 256, k >= 512) and the 2 GiB limit per tensor
    assert probe.gg_probe_gemm_kstep(224, 0, 8, 1024, 4096, 7168, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_gemm_kstep(192, 3, 8, 1024, 4096, 7168, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_gemm_kstep(192, 0, 8, 1024, 4096 + 128, 7168, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_gemm_kstep(192, 0, 8, 1024, 4096, 256, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_gemm_kstep(192, 0, 64, 8192, 4096, 7168, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_wgrad_parts(5, 8, 1000, 4096, 7168, 1, ctypes.byref(out)) != 0          # a sum that is not built
    assert probe.gg_probe_wgrad_parts(0, 8, 1000, 4096 + 64, 7168, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_wgrad_parts(0, 8, 1000, 4096, 7168 + 128, 1, ctypes.byref(out)) != 0
    assert probe.gg_probe_wgrad_parts(0, 64, 32, 4096, 7168, 1, ctypes.byref(out)) != 0           # dW beyond 4 GiB


def test_version_status_strings_and_variants(lib):
    assert gg.version() >= 100
    texts = {gg.status_str(s) for s in range(7)}
    assert len(texts) == 7 and gg.status_str(0) == "ok"
    assert gg.status_str(99) == "unknown status"
    n = gg.num_variants()
    assert n >= 1
    for v in range(n):
        assert re.fullmatch(r"\d+x\d+/\d+x\d+w/\d+s(x|-rb\w*|-k2)?", gg.variant_name(v))
    assert gg.variant_name(n) is None and gg.variant_name(-1) is None
    # the automatic choice depends on sizes only and always names a variant whose tile width divides N
    for G, M, N, K in [(8, 8192, 4096, 7168), (32, 16384, 7168, 2048), (64, 2048, 4096, 7168), (1, 1, 128, 128),
                       (0, 0, 256, 256)]:
        v = gg.auto_variant(G, M, N, K)
        assert 0 <= v < n
        assert N % int(gg.variant_name(v).split("/")[0].split("x")[1]) == 0
        vp = gg.auto_variant_padded(G, gg.padded_rows_cap(G, M), N, K)
        assert 0 <= vp < n and N % int(gg.variant_name(vp).split("/")[0].split("x")[1]) == 0
    with pytest.raises(ValueError):
        gg.auto_variant(1, 1, 100, 128)


def test_automatic_choice_on_the_four_full_size_workloads(lib):
    """The tiles the measurements of the four workloads were taken with (the choice is host arithmetic on G, M_total,
    N, K alone): a change of the estimate that moves one of them should be a decision, not an accident."""
    name = lambda G, M, N, K: gg.variant_name(gg.auto_variant(G, M, N, K))
    assert name(8, 8192, 4096, 7168) == "192x256/1x8w/3s-rb"          # gate_up
    assert name(32, 16384, 7168, 2048) == "256x256/1x8w/3s-rb"        # down
    assert name(256, 32768, 4096, 7168) == "160x256/2x4w/3s"          # many_small
    assert name(64, 2048, 4096, 7168) == "128x256/2x4w/3s"            # decode


def test_padded_rows_cap_and_workspace(lib):
    assert gg.padded_rows_cap(0, 0) == 0
    assert gg.padded_rows_cap(8, 8192) == 128 * (64 + 8)
    assert gg.padded_rows_cap(3, 1) == 128 * 4
    # the cap covers the worst case: every group one row over a multiple of 128
    for G, M in [(4, 4 * 129), (7, 5), (32, 16384)]:
        worst = sum(-(-s // 128) * 128 for s in [M // G + (1 if i < M % G else 0) for i in range(G)])
        assert gg.padded_rows_cap(G, M) >= worst
    assert gg.workspace_bytes(0, 0, 256, 256) == 0


def test_gemm_argument_validation(lib):
    f = lib.gg_fp8_grouped_gemm
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    ok_args = dict(G=2, M=100, N=256, K=256)

    def call(A=p, SA=p, B=p, SB=p, off=p, C=p, G=2, M=100, N=256, K=256):
        return f(A, SA, B, SB, off, C, G, M, N, K, p, 4096, nul)

    assert call(N=204) == GG_ERR_UNSUPPORTED      # N must be a multiple of 8 (16-byte stores of C)
    assert call(K=72) == GG_ERR_UNSUPPORTED       # K must be a multiple of 16 (16-byte fetches)
    assert call(N=0) == GG_ERR_SHAPE
    assert call(K=-128) == GG_ERR_SHAPE
    assert call(G=-1) == GG_ERR_SHAPE
    assert call(M=-1) == GG_ERR_SHAPE
    assert call(M=2 ** 31) == GG_ERR_SHAPE
    assert call(M=2 ** 31 - 1, N=2 ** 21, K=128) == GG_ERR_SHAPE      # more tiles than the kernels' 32-bit tile index
    for name in ("A", "SA", "B", "SB", "off", "C"):
        assert call(**{name: nul}) == GG_ERR_NULL, name
    # empty problems succeed without touching any pointer
    assert f(nul, nul, nul, nul, nul, nul, 0, 0, 256, 256, nul, 0, nul) == GG_OK
    assert f(nul, nul, nul, nul, nul, nul, 4, 0, 256, 256, nul, 0, nul) == GG_OK
    assert lib.gg_fp8_grouped_gemm_variant(p, p, p, p, p, p, 2, 100, 256, 256, p, 4096, nul, 999) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_grouped_gemm_padded(p, p, p, p, p, p, 2, 256, 100, 256, p, 4096, nul) == GG_ERR_UNSUPPORTED
    assert f(p, p, p, p, p, p, 2, 100, 204, 256, nul, 0, nul) == GG_ERR_UNSUPPORTED
    del ok_args


def test_pad_unpad_argument_validation(lib):
    p = ctypes.c_void_p(0x1000)
    nul = ctypes.c_void_p(0)
    cap = gg.padded_rows_cap(2, 100)
    assert lib.gg_fp8_pad(p, p, p, p, p, p, 2, 100, cap - 1, 256, nul) == GG_ERR_SHAPE
    assert lib.gg_fp8_pad(p, p, p, p, p, p, 2, 100, cap, 100, nul) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_pad(p, p, p, p, p, nul, 2, 100, cap, 256, nul) == GG_ERR_NULL
    assert lib.gg_fp8_pad(p, p, p, nul, p, p, 2, 100, cap, 256, nul) == GG_ERR_NULL
    assert lib.gg_fp8_pad(p, p, p, p, p, p, -2, 100, cap, 256, nul) == GG_ERR_SHAPE
    assert lib.gg_fp8_unpad(p, p, p, p, 2, 100, 100, nul) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_unpad(nul, p, p, p, 2, 100, 256, nul) == GG_ERR_NULL
    assert lib.gg_fp8_unpad(nul, nul, nul, nul, 0, 0, 256, nul) == GG_OK
    assert lib.gg_fp8_check_offsets(nul, 2, 100, nul) == GG_ERR_NULL


def test_ex_entry_points_validate_flags_and_sizes(lib):
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    F16, KM = binding.GG_OUT_F16, binding.GG_SA_KMAJOR
    gemm = lambda flags, M=100, N=256, K=256, A=p: lib.gg_fp8_grouped_gemm_ex(A, p, p, p, p, p, 2, M, N, K, p, 4096, nul, -1, flags)
    assert gemm(8) == GG_ERR_UNSUPPORTED and gemm(F16 | KM | 16) == GG_ERR_UNSUPPORTED      # unknown flag bits
    for flags in (0, F16, KM, F16 | KM):
        assert gemm(flags, N=204) == GG_ERR_UNSUPPORTED
        assert gemm(flags, M=-1) == GG_ERR_SHAPE
        assert gemm(flags, A=nul) == GG_ERR_NULL
        assert gemm(flags, M=0) == GG_OK
    # K-block-major scales: the K-block part of a scale's address is a 32-bit byte offset
    assert gemm(KM, M=2 ** 24, N=256, K=128 * 32) == GG_ERR_SHAPE
    cap = gg.padded_rows_cap(2, 100)
    assert lib.gg_fp8_pad_ex(p, p, p, p, p, p, 2, 100, cap, 256, nul, F16) == GG_ERR_UNSUPPORTED    # not a pad option
    assert lib.gg_fp8_pad_ex(p, p, p, p, p, p, 2, 100, cap - 1, 256, nul, KM) == GG_ERR_SHAPE
    assert lib.gg_fp8_pad_ex(p, p, p, p, p, nul, 2, 100, cap, 256, nul, KM) == GG_ERR_NULL
    assert lib.gg_fp8_quantize_rows_ex(p, nul, p, p, 10, 10, 256, nul, F16) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_quantize_rows_ex(p, nul, p, p, 10, 10, 200, nul, KM) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_quantize_rows_ex(p, nul, nul, p, 10, 10, 256, nul, KM) == GG_ERR_NULL
    assert lib.gg_fp8_quantize_rows_ex(nul, nul, nul, nul, 0, 0, 256, nul, KM) == GG_OK
    assert lib.gg_fp8_swiglu_quantize_rows_ex(p, p, p, nul, 10, 256, nul, 4) == GG_ERR_UNSUPPORTED
    assert lib.gg_fp8_swiglu_quantize_rows_ex(p, p, nul, nul, 10, 256, nul, KM) == GG_ERR_NULL
    assert lib.gg_fp8_swiglu_quantize_rows_ex(nul, nul, nul, nul, 0, 256, nul, KM) == GG_OK


def test_fused_gemm_argument_validation(lib):
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    f = lambda I=256, K=512, M=100, A2=p, variant=-1, flags=0: lib.gg_fp8_grouped_gemm_swiglu(
        p, p, p, p, p, A2, p, nul, 2, M, I, K, nul, variant, flags)
    assert f(I=192) == GG_ERR_UNSUPPORTED          # whole 128-column blocks of activations
    assert f(K=400) == GG_ERR_UNSUPPORTED and f(K=256) == GG_ERR_UNSUPPORTED    # whole K blocks, at least three
    assert f(K=384, variant=12) == GG_ERR_UNSUPPORTED    # an odd number of K blocks: the 192-row tile only
    assert f(variant=0) == GG_ERR_UNSUPPORTED and f(variant=13) == GG_ERR_UNSUPPORTED and f(variant=99) == GG_ERR_UNSUPPORTED
    assert f(flags=binding.GG_OUT_F16) == GG_ERR_UNSUPPORTED
    assert f(I=0) == GG_ERR_SHAPE and f(M=-1) == GG_ERR_SHAPE
    assert f(I=2 ** 19, K=4096) == GG_ERR_SHAPE     # an expert's weights beyond 32-bit offsets
    assert f(A2=nul) == GG_ERR_NULL
    assert f(M=0, A2=nul) == GG_OK


def test_quantize_cols_argument_validation(lib):
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    f = lambda T=256, M=256, K=128, X=p, XT=p, SX=p: lib.gg_fp8_quantize_cols(X, nul, XT, SX, T, M, K, nul)
    assert f(K=96) == GG_ERR_UNSUPPORTED and f(M=250) == GG_ERR_UNSUPPORTED
    assert f(T=-1) == GG_ERR_SHAPE and f(M=-16) == GG_ERR_SHAPE and f(K=0) == GG_ERR_SHAPE and f(K=2 ** 23) == GG_ERR_SHAPE
    assert f(X=nul) == GG_ERR_NULL and f(XT=nul) == GG_ERR_NULL and f(SX=nul) == GG_ERR_NULL
    assert f(M=0, X=nul, XT=nul, SX=nul) == GG_OK


def test_wgrad_argument_validation(lib):
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    f = lambda G=2, M=1024, N=128, K=256, XT=p, dW=p, off=p: lib.gg_fp8_grouped_gemm_wgrad(XT, p, p, p, off, dW, G, M, N, K, nul)
    assert f(M=1000 + 4) == GG_ERR_UNSUPPORTED      # the row pitch keeps every 128-token block 16-byte aligned
    assert f(N=192) == GG_ERR_UNSUPPORTED and f(K=384) == GG_ERR_UNSUPPORTED     # whole output tiles
    assert f(G=-1) == GG_ERR_SHAPE and f(M=-16) == GG_ERR_SHAPE and f(N=0) == GG_ERR_SHAPE
    assert f(M=2 ** 24, K=256) == GG_ERR_SHAPE      # K * M_total beyond 32-bit offsets
    assert f(K=2 ** 21, M=16) == GG_ERR_SHAPE
    assert f(XT=nul) == GG_ERR_NULL and f(dW=nul) == GG_ERR_NULL and f(off=nul) == GG_ERR_NULL
    assert f(G=0, XT=nul, dW=nul, off=nul) == GG_OK
    g = lambda flags: lib.gg_fp8_grouped_gemm_wgrad_ex(p, p, p, p, p, p, 0, 1024, 128, 256, nul, flags)
    assert g(8) == GG_OK and g(0) == GG_OK and g(1) == GG_ERR_UNSUPPORTED and g(8 | 2) == GG_ERR_UNSUPPORTED


def test_binding_rejects_wrong_tensors_before_calling_the_library(lib):
    import torch
    A = torch.zeros((4, 256), dtype=torch.uint8)
    SA = torch.zeros((4, 2))
    B = torch.zeros((1, 256, 256), dtype=torch.uint8)
    SB = torch.zeros((1, 2, 2))
    off = torch.tensor([0, 4], dtype=torch.int32)
    with pytest.raises(ValueError, match="GPU"):
        gg.grouped_gemm(A, SA, B, SB, off)                     # host tensors are refused: no CPU path
    with pytest.raises(TypeError):
        gg.grouped_gemm(A.float(), SA, B, SB, off)
    with pytest.raises(ValueError):
        gg.grouped_gemm(A, SA, B[:, :, :128], SB, off)
