"""ctypes binding of include/gg_fp8.h -- same names, argument marshalling only.

torch is used for device memory and streams; tensors are passed to the library
as raw device pointers.  Functions raise GGError with the library's status text
when a call returns an error code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG_DIR)
_LIB_NAME = "libgg_fp8.so"
_lib = None

GG_OK = 0


class GGError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libgg_fp8 status {status}: {text}")
        self.status = status


def library_path() -> str:
    return os.path.join(_PKG_DIR, _LIB_NAME)


HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep hipcc from forming packed-fp32 instructions on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc(src: str, out: str, verbose: bool) -> None:
    tmp = out + ".tmp"
    cmd = ["hipcc", *HIPCC_FLAGS, "-I", os.path.join(_ROOT, "include"), "-o", tmp, src]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    os.replace(tmp, out)


def build_library(verbose: bool = False) -> str:
    """Compile csrc/gg_fp8.hip (the library) and csrc/gg_probe.hip (the measurement probes of include/gg_probe.h)
    for gfx950 into the package directory (needs hipcc, no GPU).  Returns the path of the library."""
    out = library_path()
    _hipcc(os.path.join(_PKG_DIR, "csrc", "gg_fp8.hip"), out, verbose)
    _hipcc(os.path.join(_PKG_DIR, "csrc", "gg_probe.hip"), probe_library_path(), verbose)
    global _lib, _probe
    _lib = None
    _probe = None
    return out


def probe_library_path() -> str:
    return os.path.join(_PKG_DIR, "libgg_probe.so")


_probe = None


def load_probe_library() -> ctypes.CDLL:
    """The measurement probes (include/gg_probe.h); never needed by the hot path."""
    global _probe
    if _probe is not None:
        return _probe
    path = probe_library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(path)
    i32, dp = ctypes.c_int, ctypes.POINTER(ctypes.c_double)
    lib.gg_probe_mfma.restype = i32
    lib.gg_probe_mfma.argtypes = [i32, i32, i32, dp]
    lib.gg_probe_issue_mix.restype = i32
    lib.gg_probe_issue_mix.argtypes = [i32, i32, i32, i32, dp]
    lib.gg_probe_hbm.restype = i32
    lib.gg_probe_hbm.argtypes = [i32, ctypes.c_size_t, i32, dp]
    lib.gg_probe_lds_fetch.restype = i32
    lib.gg_probe_lds_fetch.argtypes = [i32, i32, i32, dp, dp]
    lib.gg_probe_gemm_kstep.restype = i32
    lib.gg_probe_gemm_kstep.argtypes = [i32, i32, i32, i32, i32, i32, i32, dp]
    lib.gg_probe_wgrad_parts.restype = i32
    lib.gg_probe_wgrad_parts.argtypes = [i32, i32, i32, i32, i32, i32, dp]
    _probe = lib
    return lib


def _probe_call(fn, *args, n_out=1):
    outs = [ctypes.c_double(0.0) for _ in range(n_out)]
    rc = fn(*args, *[ctypes.byref(o) for o in outs])
    if rc != 0:
        raise RuntimeError(f"{fn.__name__} failed with hipError_t {rc}")
    return outs[0].value if n_out == 1 else tuple(o.value for o in outs)


def probe_mfma(mode: int, data_kind: int, iters: int = 20000) -> float:
    """TFLOP/s of a register-only loop of FP8 matrix instructions (gg_probe_mfma)."""
    return _probe_call(load_probe_library().gg_probe_mfma, mode, data_kind, iters)


def probe_issue_mix(extra_salu: int, extra_valu: int, extra_lds_reads: int, iters: int = 10000) -> float:
    """TFLOP/s of the block-scaled inner loop with further instructions per matrix instruction (gg_probe_issue_mix)."""
    return _probe_call(load_probe_library().gg_probe_issue_mix, extra_salu, extra_valu, extra_lds_reads, iters)


def probe_hbm(kind: int, nbytes: int = 2 << 30, reps: int = 3) -> float:
    """GB/s of a plain HBM read (kind 0) or copy (kind 1) (gg_probe_hbm)."""
    return _probe_call(load_probe_library().gg_probe_hbm, kind, nbytes, reps)


def probe_lds_fetch(pattern: int, depth: int = 3, reps: int = 20):
    """(GB/s over the chip, bytes per clock and compute unit) of the L2 -> LDS fetch stream (gg_probe_lds_fetch)."""
    return _probe_call(load_probe_library().gg_probe_lds_fetch, pattern, depth, reps, n_out=2)


def probe_gemm_kstep(tile_rows: int, left_out: int, groups: int = 8, rows_per_group: int = 1536, n: int = 4096,
                     k: int = 7168, reps: int = 20) -> float:
    """Microseconds per launch of the second GEMM kernel with parts of its K step left out (gg_probe_gemm_kstep)."""
    return _probe_call(load_probe_library().gg_probe_gemm_kstep, tile_rows, left_out, groups, rows_per_group, n, k, reps)


def probe_wgrad_parts(left_out: int, groups: int = 8, tokens_per_group: int = 1000, n: int = 4096, k: int = 7168,
                      reps: int = 20) -> float:
    """Microseconds per launch of the weight-gradient kernel with parts of a block's work left out (gg_probe_wgrad_parts)."""
    return _probe_call(load_probe_library().gg_probe_wgrad_parts, left_out, groups, tokens_per_group, n, k, reps)


def load_library() -> ctypes.CDLL:
    """Load the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no CPU fallback for libgg_fp8)")
    lib = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    lib.gg_fp8_version.restype = i32
    lib.gg_fp8_version.argtypes = []
    lib.gg_fp8_status_str.restype = ctypes.c_char_p
    lib.gg_fp8_status_str.argtypes = [i32]
    lib.gg_fp8_workspace_bytes.restype = sz
    lib.gg_fp8_workspace_bytes.argtypes = [i32, i64, i32, i32]
    lib.gg_fp8_workspace_bytes_variant.restype = sz
    lib.gg_fp8_workspace_bytes_variant.argtypes = [i32, i64, i32, i32, i32]
    lib.gg_fp8_grouped_gemm.restype = i32
    lib.gg_fp8_grouped_gemm.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, sz, vp]
    lib.gg_fp8_grouped_gemm_variant.restype = i32
    lib.gg_fp8_grouped_gemm_variant.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, sz, vp, i32]
    lib.gg_fp8_num_variants.restype = i32
    lib.gg_fp8_grouped_gemm_f16.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, sz, vp, i32]
    lib.gg_fp8_grouped_gemm_f16.restype = i32
    lib.gg_fp8_grouped_gemm_ex.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, sz, vp, i32, ctypes.c_uint]
    lib.gg_fp8_grouped_gemm_ex.restype = i32
    lib.gg_fp8_grouped_gemm_splitk_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, i32, ctypes.c_uint]
    lib.gg_fp8_grouped_gemm_splitk_noalloc.restype = i32
    lib.gg_fp8_noalloc_max_elements.argtypes = []
    lib.gg_fp8_noalloc_max_elements.restype = sz
    lib.gg_fp8_grouped_gemm_swiglu.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, i32, ctypes.c_uint]
    lib.gg_fp8_grouped_gemm_swiglu.restype = i32
    lib.gg_fp8_grouped_gemm_wgrad.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp]
    lib.gg_fp8_grouped_gemm_wgrad.restype = i32
    lib.gg_fp8_grouped_gemm_wgrad_ex.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, ctypes.c_uint]
    lib.gg_fp8_grouped_gemm_wgrad_ex.restype = i32
    lib.gg_fp8_quantize_cols.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp]
    lib.gg_fp8_quantize_cols.restype = i32
    lib.gg_fp8_pad_ex.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, vp, ctypes.c_uint]
    lib.gg_fp8_pad_ex.restype = i32
    lib.gg_fp8_quantize_rows_ex.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, ctypes.c_uint]
    lib.gg_fp8_quantize_rows_ex.restype = i32
    lib.gg_fp8_swiglu_quantize_rows_ex.argtypes = [vp, vp, vp, vp, i64, i32, vp, ctypes.c_uint]
    lib.gg_fp8_swiglu_quantize_rows_ex.restype = i32
    lib.gg_fp8_num_variants.argtypes = []
    lib.gg_fp8_variant_name.restype = ctypes.c_char_p
    lib.gg_fp8_variant_name.argtypes = [i32]
    lib.gg_fp8_auto_variant.restype = i32
    lib.gg_fp8_auto_variant.argtypes = [i32, i64, i32, i32]
    lib.gg_fp8_auto_variant_padded.restype = i32
    lib.gg_fp8_auto_variant_padded.argtypes = [i32, i64, i32, i32]
    lib.gg_fp8_padded_rows_cap.restype = i64
    lib.gg_fp8_padded_rows_cap.argtypes = [i32, i64]
    lib.gg_fp8_pad.restype = i32
    lib.gg_fp8_pad.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, vp]
    lib.gg_fp8_grouped_gemm_padded.restype = i32
    lib.gg_fp8_grouped_gemm_padded.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, vp, sz, vp]
    lib.gg_fp8_unpad.restype = i32
    lib.gg_fp8_unpad.argtypes = [vp, vp, vp, vp, i32, i64, i32, vp]
    lib.gg_fp8_check_offsets.restype = i32
    lib.gg_fp8_quantize_rows.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp]
    lib.gg_fp8_quantize_rows.restype = i32
    lib.gg_fp8_swiglu_quantize_rows.argtypes = [vp, vp, vp, vp, i64, i32, vp]
    lib.gg_fp8_swiglu_quantize_rows.restype = i32
    lib.gg_fp8_check_offsets.argtypes = [vp, i32, i64, vp]
    _lib = lib
    return lib


EXPORTED_SYMBOLS = [
    "gg_fp8_version", "gg_fp8_status_str", "gg_fp8_workspace_bytes", "gg_fp8_workspace_bytes_variant", "gg_fp8_grouped_gemm",
    "gg_fp8_grouped_gemm_variant", "gg_fp8_grouped_gemm_f16", "gg_fp8_grouped_gemm_ex", "gg_fp8_num_variants", "gg_fp8_variant_name", "gg_fp8_auto_variant", "gg_fp8_auto_variant_padded", "gg_fp8_padded_rows_cap",
    "gg_fp8_pad", "gg_fp8_grouped_gemm_padded", "gg_fp8_unpad", "gg_fp8_quantize_rows", "gg_fp8_swiglu_quantize_rows", "gg_fp8_check_offsets",
    "gg_fp8_grouped_gemm_splitk_noalloc", "gg_fp8_noalloc_max_elements", "gg_fp8_pad_ex", "gg_fp8_quantize_rows_ex", "gg_fp8_swiglu_quantize_rows_ex", "gg_fp8_grouped_gemm_swiglu",
    "gg_fp8_grouped_gemm_wgrad", "gg_fp8_grouped_gemm_wgrad_ex", "gg_fp8_quantize_cols",
]


# ---------------------------------------------------------------------------- helpers
def _check(status: int):
    if status != GG_OK:
        raise GGError(status, status_str(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _want(t, name, dtype, ndim):
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions, got {t.dim()}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")


GG_OUT_F16, GG_SA_KMAJOR, GG_PADDED_GROUPS, GG_OUT_BF16 = 1, 2, 4, 8        # flags of the _ex entry points


def _gemm_shapes(A, SA, B, SB, group_offsets, sa_kmajor=False):
    _want(A, "A", torch.uint8, 2)
    _want(SA, "SA", torch.float32, 2)
    _want(B, "B", torch.uint8, 3)
    _want(SB, "SB", torch.float32, 3)
    _want(group_offsets, "group_offsets", torch.int32, 1)
    M_total, K = A.shape
    G, N, K2 = B.shape
    if K2 != K:
        raise ValueError(f"A has K={K} but B has K={K2}")
    if group_offsets.shape[0] != G + 1:
        raise ValueError(f"group_offsets must have G+1={G + 1} entries")
    KB, NB = -(-K // 128), -(-N // 128)          # ceilings (Table 1 of the paper)
    sa_shape = (KB, M_total) if sa_kmajor else (M_total, KB)
    if tuple(SA.shape) != sa_shape:
        raise ValueError(f"SA must be {list(sa_shape)}")
    if tuple(SB.shape) != (G, NB, KB):
        raise ValueError(f"SB must be [{G}, {NB}, {KB}]")
    return G, M_total, N, K


# ---------------------------------------------------------------------------- the API
def version() -> int:
    return load_library().gg_fp8_version()


def status_str(status: int) -> str:
    return load_library().gg_fp8_status_str(int(status)).decode()


def workspace_bytes(G: int, M_total: int, N: int, K: int, variant: int = -1) -> int:
    """gg_fp8_workspace_bytes (variant = -1: the automatic choice) / gg_fp8_workspace_bytes_variant."""
    return int(load_library().gg_fp8_workspace_bytes_variant(G, M_total, N, K, int(variant)))


def num_variants() -> int:
    return load_library().gg_fp8_num_variants()


def auto_variant_padded(G: int, M_pad_cap: int, N: int, K: int) -> int:
    """Index of the variant gg_fp8_grouped_gemm_padded (or GG_PADDED_GROUPS with variant = -1) uses."""
    v = load_library().gg_fp8_auto_variant_padded(G, M_pad_cap, N, K)
    if v < 0:
        raise ValueError(f"gg_fp8_auto_variant_padded: {status_str(-v)}")
    return v


def auto_variant(G: int, M_total: int, N: int, K: int) -> int:
    """Index of the variant grouped_gemm(variant=-1) uses for these sizes."""
    v = load_library().gg_fp8_auto_variant(G, M_total, N, K)
    if v < 0:
        raise ValueError(f"gg_fp8_auto_variant: {status_str(-v)}")
    return v


def variant_name(v: int):
    s = load_library().gg_fp8_variant_name(v)
    return None if s is None else s.decode()


_ws_cache = {}


def _workspace(G, M_total, N, K, device, workspace=None, stream=None, variant=-1):
    """The scratch buffer of a GEMM call: the caller's, or one per (device, stream) kept by this binding (calls on one
    stream run in order, so they may share it; the library clears what it uses at the start of every call)."""
    n = workspace_bytes(G, M_total, N, K, variant)
    if workspace is not None:
        _want(workspace, "workspace", torch.uint8, 1)
        if workspace.numel() < n:
            raise ValueError(f"workspace must hold at least {n} bytes")
        return workspace, workspace.numel()
    if n == 0:
        return None, 0
    key = (device, (stream if stream is not None else torch.cuda.current_stream(device)).cuda_stream)
    ws = _ws_cache.get(key)
    if ws is None or ws.numel() < n:
        ws = _ws_cache[key] = torch.zeros(n, dtype=torch.uint8, device=device)
    return ws, ws.numel()


def grouped_gemm(A, SA, B, SB, group_offsets, C=None, variant: int = -1, stream=None, out_dtype=None, sa_kmajor=False,
                 workspace=None):
    """C[r, :] = round(block-scaled A[r, :] @ B[g]^T) for every row r of every group g (gg_fp8_grouped_gemm_variant,
    gg_fp8_grouped_gemm_f16 when C / out_dtype is torch.float16, gg_fp8_grouped_gemm_ex when sa_kmajor).

    A uint8 [M_total, K] (e4m3 bytes), SA float32 [M_total, K/128] (sa_kmajor: [K/128, M_total]), B uint8 [G, N, K],
    SB float32 [G, N/128, K/128], group_offsets int32 [G+1]; returns C bfloat16 (default) or float16 [M_total, N]
    (allocated here unless given; rows outside the groups are left as they are).  With variant = -1, row-major
    scales and bfloat16 output this is the plain gg_fp8_grouped_gemm call.  workspace: uint8 tensor of at least
    workspace_bytes(...) bytes (default: one kept per stream by this binding).
    """
    lib = load_library()
    G, M_total, N, K = _gemm_shapes(A, SA, B, SB, group_offsets, sa_kmajor)
    if out_dtype is None:
        out_dtype = C.dtype if C is not None else torch.bfloat16
    if out_dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("C must be bfloat16 or float16")
    if C is None:
        C = torch.empty((M_total, N), dtype=out_dtype, device=A.device)
    _want(C, "C", out_dtype, 2)
    if tuple(C.shape) != (M_total, N):
        raise ValueError(f"C must be [{M_total}, {N}]")
    ws, n = _workspace(G, M_total, N, K, A.device, workspace, stream, variant)
    args = (_ptr(A), _ptr(SA), _ptr(B), _ptr(SB), _ptr(group_offsets), _ptr(C), G, M_total, N, K, _ptr(ws), n,
            _stream(stream), int(variant))
    if variant == -1 and not sa_kmajor and out_dtype == torch.bfloat16:
        _check(lib.gg_fp8_grouped_gemm(*args[:-1]))
    elif sa_kmajor:
        _check(lib.gg_fp8_grouped_gemm_ex(*args, GG_SA_KMAJOR | (GG_OUT_F16 if out_dtype == torch.float16 else 0)))
    else:
        _check((lib.gg_fp8_grouped_gemm_f16 if out_dtype == torch.float16 else lib.gg_fp8_grouped_gemm_variant)(*args))
    return C


def grouped_gemm_splitk_noalloc(A, SA, B, SB, group_offsets, C, variant: int = -1, stream=None, sa_kmajor=False):
    """gg_fp8_grouped_gemm_splitk_noalloc: the split-K GEMM on the library's built-in scratch (no workspace, no
    allocation in the library; C must be given).  M_total * N <= noalloc_max_elements()."""
    lib = load_library()
    G, M_total, N, K = _gemm_shapes(A, SA, B, SB, group_offsets, sa_kmajor)
    if C.dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("C must be bfloat16 or float16")
    _want(C, "C", C.dtype, 2)
    if tuple(C.shape) != (M_total, N):
        raise ValueError(f"C must be [{M_total}, {N}]")
    flags = (GG_SA_KMAJOR if sa_kmajor else 0) | (GG_OUT_F16 if C.dtype == torch.float16 else 0)
    _check(lib.gg_fp8_grouped_gemm_splitk_noalloc(_ptr(A), _ptr(SA), _ptr(B), _ptr(SB), _ptr(group_offsets), _ptr(C),
                                                  G, M_total, N, K, _stream(stream), int(variant), flags))
    return C


def noalloc_max_elements() -> int:
    return int(load_library().gg_fp8_noalloc_max_elements())


def grouped_gemm_swiglu(A, SA, B, SB, group_offsets, A2=None, SA2=None, act_out=None, want_act=False, variant: int = -1,
                        stream=None, sa_kmajor=False):
    """gg_fp8_grouped_gemm_swiglu: the grouped GEMM with B [G, 2I, K] (gate rows, then up rows), silu(gate) * up and
    the 1x128 quantiser in one kernel: returns (A2 uint8 [M_total, I], SA2 float32 [M_total, I/128] or
    [I/128, M_total] with sa_kmajor, act bf16 [M_total, I] or None)."""
    lib = load_library()
    G, M_total, N, K = _gemm_shapes(A, SA, B, SB, group_offsets, sa_kmajor)
    if N % 2:
        raise ValueError("B must hold an even number of rows per group (gate | up)")
    inter = N // 2
    if A2 is None:
        A2 = torch.empty((M_total, inter), dtype=torch.uint8, device=A.device)
    if SA2 is None:
        SA2 = torch.empty((inter // 128, M_total) if sa_kmajor else (M_total, inter // 128), dtype=torch.float32, device=A.device)
    if act_out is None and want_act:
        act_out = torch.empty((M_total, inter), dtype=torch.bfloat16, device=A.device)
    _want(A2, "A2", torch.uint8, 2)
    _want(SA2, "SA2", torch.float32, 2)
    if act_out is not None:
        _want(act_out, "act_out", torch.bfloat16, 2)
        if tuple(act_out.shape) != (M_total, inter):
            raise ValueError(f"act_out must be [{M_total}, {inter}]")
    if tuple(A2.shape) != (M_total, inter) or tuple(SA2.shape) != ((inter // 128, M_total) if sa_kmajor else (M_total, inter // 128)):
        raise ValueError("A2 or SA2 does not have the shape of the output")
    _check(lib.gg_fp8_grouped_gemm_swiglu(_ptr(A), _ptr(SA), _ptr(B), _ptr(SB), _ptr(group_offsets), _ptr(A2), _ptr(SA2),
                                          _ptr(act_out), G, M_total, inter, K, _stream(stream), int(variant),
                                          GG_SA_KMAJOR if sa_kmajor else 0))
    return A2, SA2, act_out


def grouped_gemm_wgrad(XT, SX, DYT, SDY, group_offsets, dW=None, stream=None, out_bf16=False):
    """gg_fp8_grouped_gemm_wgrad(_ex): dW [G, N, K] float32 (bfloat16 with out_bf16) from XT uint8 [K, M_total], SX
    float32 [ceil(M_total/128), K], DYT uint8 [N, M_total], SDY float32 [ceil(M_total/128), N] and int32 group_offsets
    [G+1] (tokens of group g)."""
    lib = load_library()
    _want(XT, "XT", torch.uint8, 2)
    _want(DYT, "DYT", torch.uint8, 2)
    _want(SX, "SX", torch.float32, 2)
    _want(SDY, "SDY", torch.float32, 2)
    _want(group_offsets, "group_offsets", torch.int32, 1)
    K, M_total = XT.shape
    N = DYT.shape[0]
    MB = (M_total + 127) // 128
    G = group_offsets.shape[0] - 1
    if DYT.shape[1] != M_total or tuple(SX.shape) != (MB, K) or tuple(SDY.shape) != (MB, N):
        raise ValueError("XT [K, M_total], DYT [N, M_total], SX [ceil(M_total/128), K], SDY [ceil(M_total/128), N] expected")
    for t, name in ((XT, "XT"), (SX, "SX"), (DYT, "DYT"), (SDY, "SDY"), (group_offsets, "group_offsets")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous device tensor")
    out_dtype = torch.bfloat16 if out_bf16 else torch.float32
    if dW is None:
        dW = torch.empty((G, N, K), dtype=out_dtype, device=XT.device)
    _want(dW, "dW", out_dtype, 3)
    if tuple(dW.shape) != (G, N, K) or not dW.is_cuda or not dW.is_contiguous():
        raise ValueError(f"dW must be a contiguous device tensor [{G}, {N}, {K}]")
    args = (_ptr(XT), _ptr(SX), _ptr(DYT), _ptr(SDY), _ptr(group_offsets), _ptr(dW), G, M_total, N, K, _stream(stream))
    _check(lib.gg_fp8_grouped_gemm_wgrad_ex(*args, GG_OUT_BF16) if out_bf16 else lib.gg_fp8_grouped_gemm_wgrad(*args))
    return dW


def quantize_cols(X, row_src=None, M_total=None, XT=None, SX=None, stream=None):
    """gg_fp8_quantize_cols: X [T, K] bf16 -> (XT uint8 [K, M_total], SX float32 [ceil(M_total/128), K]): the block
    quantiser along the tokens, transposed; output token r is input row row_src[r] (int32 [M_total] on the device;
    None = identity)."""
    lib = load_library()
    _want(X, "X", torch.bfloat16, 2)
    T, K = X.shape
    if row_src is not None:
        _want(row_src, "row_src", torch.int32, 1)
        M_total = row_src.shape[0]
    elif M_total is None:
        M_total = T
    MB = (M_total + 127) // 128
    if XT is None:
        XT = torch.empty((K, M_total), dtype=torch.uint8, device=X.device)
    if SX is None:
        SX = torch.empty((MB, K), dtype=torch.float32, device=X.device)
    _want(XT, "XT", torch.uint8, 2)
    _want(SX, "SX", torch.float32, 2)
    if tuple(XT.shape) != (K, M_total) or tuple(SX.shape) != (MB, K):
        raise ValueError("XT or SX does not have the shape of the output")
    _check(lib.gg_fp8_quantize_cols(_ptr(X), _ptr(row_src), _ptr(XT), _ptr(SX), T, M_total, K, _stream(stream)))
    return XT, SX


def padded_rows_cap(G: int, M_total: int) -> int:
    return int(load_library().gg_fp8_padded_rows_cap(G, M_total))


def pad(A, SA, group_offsets, M_pad_cap: int | None = None, stream=None, sa_kmajor=False, A_pad=None, SA_pad=None):
    """gg_fp8_pad (gg_fp8_pad_ex when sa_kmajor: SA [K/128, M_total] -> SA_pad [K/128, M_pad_cap]): returns
    (A_pad, SA_pad, padded_offsets) with every group at a multiple of 128 rows.  Rows past the last padded group are
    not written (the buffers come from torch.empty unless the caller passes A_pad and SA_pad)."""
    lib = load_library()
    _want(A, "A", torch.uint8, 2)
    _want(SA, "SA", torch.float32, 2)
    _want(group_offsets, "group_offsets", torch.int32, 1)
    M_total, K = A.shape
    G = group_offsets.shape[0] - 1
    if M_pad_cap is None:
        M_pad_cap = padded_rows_cap(G, M_total)
    KB = -(-K // 128)
    if tuple(SA.shape) != ((KB, M_total) if sa_kmajor else (M_total, KB)):
        raise ValueError("SA does not have the shape of its storage order")
    sa_pad_shape = (KB, M_pad_cap) if sa_kmajor else (M_pad_cap, KB)
    if A_pad is None:
        A_pad = torch.empty((M_pad_cap, K), dtype=torch.uint8, device=A.device)
    if SA_pad is None:
        SA_pad = torch.empty(sa_pad_shape, dtype=torch.float32, device=A.device)
    _want(A_pad, "A_pad", torch.uint8, 2)
    _want(SA_pad, "SA_pad", torch.float32, 2)
    if tuple(A_pad.shape) != (M_pad_cap, K) or tuple(SA_pad.shape) != sa_pad_shape:
        raise ValueError("A_pad / SA_pad do not have M_pad_cap rows of the inputs' width")
    poff = torch.empty(G + 1, dtype=torch.int32, device=A.device)
    args = (_ptr(A), _ptr(SA), _ptr(group_offsets), _ptr(A_pad), _ptr(SA_pad), _ptr(poff), G, M_total, M_pad_cap, K,
            _stream(stream))
    _check(lib.gg_fp8_pad_ex(*args, GG_SA_KMAJOR) if sa_kmajor else lib.gg_fp8_pad(*args))
    return A_pad, SA_pad, poff


def grouped_gemm_padded(A_pad, SA_pad, B, SB, padded_offsets, C_pad=None, stream=None, sa_kmajor=False):
    """gg_fp8_grouped_gemm_padded: the same GEMM on the 128-aligned problem; returns C_pad.  (sa_kmajor: the same
    through gg_fp8_grouped_gemm_ex, as the header prescribes.)"""
    lib = load_library()
    if sa_kmajor:
        G, M_pad_cap, N, K = _gemm_shapes(A_pad, SA_pad, B, SB, padded_offsets, True)
        if C_pad is None:
            C_pad = torch.empty((M_pad_cap, N), dtype=torch.bfloat16, device=A_pad.device)
        _want(C_pad, "C_pad", torch.bfloat16, 2)
        ws, n = _workspace(G, M_pad_cap, N, K, A_pad.device, None, stream)
        _check(lib.gg_fp8_grouped_gemm_ex(_ptr(A_pad), _ptr(SA_pad), _ptr(B), _ptr(SB), _ptr(padded_offsets), _ptr(C_pad),
                                          G, M_pad_cap, N, K, _ptr(ws), n, _stream(stream), -1,
                                          GG_SA_KMAJOR | GG_PADDED_GROUPS))
        return C_pad
    G, M_pad_cap, N, K = _gemm_shapes(A_pad, SA_pad, B, SB, padded_offsets)
    if C_pad is None:
        C_pad = torch.empty((M_pad_cap, N), dtype=torch.bfloat16, device=A_pad.device)
    _want(C_pad, "C_pad", torch.bfloat16, 2)
    ws, n = _workspace(G, M_pad_cap, N, K, A_pad.device, None, stream)
    _check(lib.gg_fp8_grouped_gemm_padded(_ptr(A_pad), _ptr(SA_pad), _ptr(B), _ptr(SB), _ptr(padded_offsets),
                                          _ptr(C_pad), G, M_pad_cap, N, K, _ptr(ws), n, _stream(stream)))
    return C_pad


def unpad(C_pad, group_offsets, padded_offsets, M_total: int, C=None, stream=None):
    """gg_fp8_unpad: gathers the valid rows of C_pad into C [M_total, N]."""
    lib = load_library()
    _want(C_pad, "C_pad", torch.bfloat16, 2)
    N = C_pad.shape[1]
    G = group_offsets.shape[0] - 1
    if C is None:
        C = torch.empty((M_total, N), dtype=torch.bfloat16, device=C_pad.device)
    _check(lib.gg_fp8_unpad(_ptr(C_pad), _ptr(group_offsets), _ptr(padded_offsets), _ptr(C), G, M_total, N,
                            _stream(stream)))
    return C


def quantize_rows(X, row_src=None, M_total=None, A=None, SA=None, stream=None, sa_kmajor=False):
    """gg_fp8_quantize_rows(_ex): X [T, K] bf16 -> (A uint8 [M_total, K], SA float32 [M_total, K/128], or
    [K/128, M_total] with sa_kmajor); output row r is input row row_src[r] (int32 [M_total] on the device;
    None = identity)."""
    lib = load_library()
    _want(X, "X", torch.bfloat16, 2)
    T, K = X.shape
    if row_src is not None:
        _want(row_src, "row_src", torch.int32, 1)
        M_total = row_src.shape[0]
    elif M_total is None:
        M_total = T
    if A is None:
        A = torch.empty((M_total, K), dtype=torch.uint8, device=X.device)
    if SA is None:
        SA = torch.empty((K // 128, M_total) if sa_kmajor else (M_total, K // 128), dtype=torch.float32, device=X.device)
    _want(A, "A", torch.uint8, 2)
    _want(SA, "SA", torch.float32, 2)
    if tuple(SA.shape) != ((K // 128, M_total) if sa_kmajor else (M_total, K // 128)) or tuple(A.shape) != (M_total, K):
        raise ValueError("A or SA does not have the shape of the output")
    args = (_ptr(X), _ptr(row_src), _ptr(A), _ptr(SA), T, M_total, K, _stream(stream))
    _check(lib.gg_fp8_quantize_rows_ex(*args, GG_SA_KMAJOR) if sa_kmajor else lib.gg_fp8_quantize_rows(*args))
    return A, SA


def swiglu_quantize_rows(H, A=None, SA=None, act_out=None, want_act=False, stream=None, sa_kmajor=False):
    """gg_fp8_swiglu_quantize_rows(_ex): H [M, 2I] bf16 -> (A uint8 [M, I], SA float32 [M, I/128], or [I/128, M] with
    sa_kmajor, act bf16 [M, I] or None)."""
    lib = load_library()
    _want(H, "H", torch.bfloat16, 2)
    M, two_i = H.shape
    if two_i % 2:
        raise ValueError("H must have an even number of columns")
    inter = two_i // 2
    if A is None:
        A = torch.empty((M, inter), dtype=torch.uint8, device=H.device)
    if SA is None:
        SA = torch.empty((inter // 128, M) if sa_kmajor else (M, inter // 128), dtype=torch.float32, device=H.device)
    if act_out is None and want_act:
        act_out = torch.empty((M, inter), dtype=torch.bfloat16, device=H.device)
    _want(A, "A", torch.uint8, 2)
    _want(SA, "SA", torch.float32, 2)
    if act_out is not None:
        _want(act_out, "act_out", torch.bfloat16, 2)
    if tuple(SA.shape) != ((inter // 128, M) if sa_kmajor else (M, inter // 128)) or tuple(A.shape) != (M, inter):
        raise ValueError("A or SA does not have the shape of the output")
    args = (_ptr(H), _ptr(A), _ptr(SA), _ptr(act_out), M, inter, _stream(stream))
    _check(lib.gg_fp8_swiglu_quantize_rows_ex(*args, GG_SA_KMAJOR) if sa_kmajor else lib.gg_fp8_swiglu_quantize_rows(*args))
    return A, SA, act_out


def check_offsets(group_offsets, M_total: int, stream=None) -> int:
    """gg_fp8_check_offsets (debug; synchronises): returns the status instead of raising."""
    lib = load_library()
    G = group_offsets.shape[0] - 1
    return lib.gg_fp8_check_offsets(_ptr(group_offsets), G, M_total, _stream(stream))
