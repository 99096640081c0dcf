#!/usr/bin/env python3
"""The paper's parameter sweep (Sec. 3.1, App. C.1) on one MI355X: padding-free grouped GEMM against
pad-then-GEMM over N, K in {3072..8192}, G in {4, 8, 16, 32}, M in {8192..65536}, with group sizes drawn by the
paper's generator.  Inputs are seeded and synthetic; both paths run the library's own kernels (the pad path is
pad kernels + the same GEMM on 128-aligned offsets + optional unpad), so the comparison isolates padding.

    python sweep.py                      # full grid (576 points), JSON lines to stdout, summary to stderr
    python sweep.py --grid quick         # the 16 corner points
    python sweep.py --out sweep.jsonl --summary sweep.md

Per point: time per launch of the three paths (HIP events on the launch stream; same buffers every launch, so small
problems are served by the Infinity Cache in all three paths alike, unless --cold flushes the caches before every
timed launch), TFLOP/s on valid rows, speed-up, and
the memory the row tensors save (1 - M / M_pad, the quantity whose magnitude the paper's abstract quotes).
The summary lists ranges and the Pearson correlations the paper discusses in Sec. 3.2 (speed-up against N, K, M,
G, M/G; memory saving against M/G).
"""
import argparse
import ctypes
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--grid", choices=["full", "quick"], default="full")
    ap.add_argument("--Ns", type=str, default=None, help="comma-separated override of the N values")
    ap.add_argument("--Ks", type=str, default=None)
    ap.add_argument("--Gs", type=str, default=None)
    ap.add_argument("--Ms", type=str, default=None)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--variant", type=int, default=-1, help="tile variant for every GEMM launch (-1: automatic)")
    ap.add_argument("--cold", action="store_true",
                    help="overwrite a 1 GiB buffer before every timed launch, so that neither the L2s nor the 256 MB "
                         "Infinity Cache hold any input (default: same buffers every launch, caches warm)")
    ap.add_argument("--free-only", action="store_true",
                    help="time the padding-free path only (for comparing tile variants; the pad columns repeat its time)")
    ap.add_argument("--sa-layout", choices=["kmajor", "row"], default="kmajor",
                    help="storage order of the activation scales: [K/128, M] (GG_SA_KMAJOR, default) or [M, K/128]")
    ap.add_argument("--seed", type=int, default=20250816)
    ap.add_argument("--out", type=str, default=None, help="write the JSON lines here instead of stdout")
    ap.add_argument("--summary", type=str, default=None, help="write the summary (markdown) here as well as to stderr")
    args = ap.parse_args()

    import torch
    import paper_2508_16584_amd as gg
    from workloads.configs import paper_group_sizes
    from workloads.quantize import quantize_a, quantize_b

    if not torch.cuda.is_available():
        sys.exit("sweep.py needs an MI355X: no GPU visible")
    dev = torch.device("cuda:0")
    lib = gg.load_library()

    full = [3072, 4096, 5120, 6144, 7168, 8192]
    if args.grid == "full":
        Ns, Ks, Gs, Ms = full, full, [4, 8, 16, 32], [8192, 16384, 32768, 65536]
    else:
        Ns, Ks, Gs, Ms = [3072, 8192], [3072, 8192], [4, 32], [8192, 65536]
    pick = lambda s, d: [int(x) for x in s.split(",")] if s else d
    Ns, Ks, Gs, Ms = pick(args.Ns, Ns), pick(args.Ks, Ks), pick(args.Gs, Gs), pick(args.Ms, Ms)
    Gmax, Mmax = max(Gs), max(Ms)

    flags = 2 if args.sa_layout == "kmajor" else 0        # GG_SA_KMAJOR
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # bring the GPU to its sustained clock before the first grid point (about 150 ms of matrix work)
    wu = torch.randn((4096, 4096), device=dev, dtype=torch.bfloat16)
    t_wu = time.perf_counter()
    while time.perf_counter() - t_wu < 0.15:
        for _ in range(10):
            wu @ wu
        torch.cuda.synchronize()
    del wu
    sink = open(args.out, "w") if args.out else sys.stdout
    rows_out = []
    t_start = time.perf_counter()

    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if args.cold else None

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        if flush is None:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps        # ms per launch
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in ev:
            flush.fill_(1)
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev]))

    point = 0
    for K in Ks:
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed + K)
        # activations for the largest M of the grid (any prefix of i.i.d. rows is a valid smaller problem)
        A = torch.empty((Mmax, K), dtype=torch.uint8, device=dev)
        SA = torch.empty((Mmax, K // 128), dtype=torch.float32, device=dev)
        for r0 in range(0, Mmax, 8192):
            rows = min(8192, Mmax - r0)
            x = torch.randn((rows, K), generator=gen, device=dev, dtype=torch.float32)
            A[r0:r0 + rows], SA[r0:r0 + rows] = quantize_a(x)
        for N in Ns:
            B = torch.empty((Gmax, N, K), dtype=torch.uint8, device=dev)
            SB = torch.empty((Gmax, N // 128, K // 128), dtype=torch.float32, device=dev)
            for g in range(Gmax):
                w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
                B[g], SB[g] = quantize_b(w)
            C = torch.empty((Mmax, N), dtype=torch.bfloat16, device=dev)
            ws = torch.zeros(max(gg.workspace_bytes(Gmax, Mmax, N, K), 4), dtype=torch.uint8, device=dev)
            cap_max = gg.padded_rows_cap(Gmax, Mmax)
            A_pad = torch.empty((cap_max, K), dtype=torch.uint8, device=dev)
            SA_pad = torch.empty((cap_max, K // 128), dtype=torch.float32, device=dev)
            C_pad = torch.empty((cap_max, N), dtype=torch.bfloat16, device=dev)
            for G in Gs:
                for M in Ms:
                    rng = np.random.default_rng([args.seed, N, K, G, M])
                    sizes = paper_group_sizes(M, G, rng)
                    off_h = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
                    off = torch.from_numpy(off_h).to(dev)
                    poff = torch.empty(G + 1, dtype=torch.int32, device=dev)
                    cap = gg.padded_rows_cap(G, M)
                    # the scales of the first M rows in the chosen order (SA_pad is written in the same order)
                    SA_M = SA[:M].t().contiguous() if flags else SA

                    def free_step():
                        rc = lib.gg_fp8_grouped_gemm_ex(vp(A), vp(SA_M), vp(B), vp(SB), vp(off), vp(C), G, M, N, K,
                                                        vp(ws), ws.numel(), stream, args.variant, flags)
                        assert rc == 0, gg.status_str(rc)

                    def pad_step(with_unpad):
                        rc = lib.gg_fp8_pad_ex(vp(A), vp(SA_M), vp(off), vp(A_pad), vp(SA_pad), vp(poff), G, M, cap, K, stream, flags)
                        rc |= lib.gg_fp8_grouped_gemm_ex(vp(A_pad), vp(SA_pad), vp(B), vp(SB), vp(poff), vp(C_pad),
                                                         G, cap, N, K, vp(ws), ws.numel(), stream, args.variant,
                                                         flags | (4 if args.variant < 0 else 0))      # GG_PADDED_GROUPS
                        if with_unpad:
                            rc |= lib.gg_fp8_unpad(vp(C_pad), vp(off), vp(poff), vp(C), G, M, N, stream)
                        assert rc == 0

                    t_free = timed(free_step)
                    m_pad = int(np.sum(128 * ((sizes + 127) // 128)))
                    if args.free_only:
                        t_pad = t_pad_unpad = t_free
                    else:
                        t_pad = timed(lambda: pad_step(False))
                        t_pad_unpad = timed(lambda: pad_step(True))
                        assert m_pad == int(poff[-1].item())
                    used = args.variant if args.variant >= 0 else gg.auto_variant(G, M, N, K)
                    rec = {
                        "N": N, "K": K, "G": G, "M": M, "M_pad": m_pad,
                        "rows_min": int(sizes.min()), "rows_max": int(sizes.max()),
                        "variant": gg.variant_name(used),
                        "t_free_us": round(t_free * 1e3, 2), "t_pad_gemm_us": round(t_pad * 1e3, 2),
                        "t_pad_gemm_unpad_us": round(t_pad_unpad * 1e3, 2),
                        "tflops": round(2.0 * M * N * K / (t_free * 1e-3) / 1e12, 1),
                        "speedup_vs_pad_gemm": round(t_pad / t_free, 4),
                        "speedup_vs_pad_gemm_unpad": round(t_pad_unpad / t_free, 4),
                        "mem_saving_row_tensors": round(1.0 - M / m_pad, 4),
                    }
                    rows_out.append(rec)
                    sink.write(json.dumps(rec) + "\n")
                    sink.flush()
                    point += 1
                    if point % 16 == 0:
                        print(f"[sweep] {point} points, {time.perf_counter() - t_start:.0f} s", file=sys.stderr, flush=True)
            del B, SB, C, A_pad, SA_pad, C_pad
        del A, SA
        torch.cuda.empty_cache()

    # ---- summary -----------------------------------------------------------------------------------------
    def col(name):
        return np.array([r[name] for r in rows_out], dtype=np.float64)

    def corr(x, y):
        return float(np.corrcoef(x, y)[0, 1]) if len(x) > 2 and np.std(x) > 0 and np.std(y) > 0 else float("nan")

    sp, spu, mem, tf = col("speedup_vs_pad_gemm"), col("speedup_vs_pad_gemm_unpad"), col("mem_saving_row_tensors"), col("tflops")
    Nc, Kc, Gc, Mc = col("N"), col("K"), col("G"), col("M")
    lines = [
        f"points: {len(rows_out)}  (N in {Ns}, K in {Ks}, G in {Gs}, M in {Ms}; variant {'auto' if args.variant < 0 else args.variant}; "
        f"activation scales {'K-block-major' if flags else 'row-major'}; caches {'flushed before every launch' if args.cold else 'warm'})",
        f"TFLOP/s on valid rows: min {tf.min():.0f}  median {np.median(tf):.0f}  max {tf.max():.0f}",
        f"speed-up over pad+GEMM: min {sp.min():.3f}  median {np.median(sp):.3f}  max {sp.max():.3f}",
        f"speed-up over pad+GEMM+unpad: min {spu.min():.3f}  median {np.median(spu):.3f}  max {spu.max():.3f}",
        f"memory saved on the row tensors (1 - M/M_pad): min {mem.min():.3f}  median {np.median(mem):.3f}  max {mem.max():.3f}",
        "Pearson r of the speed-up over pad+GEMM with N: %.3f, K: %.3f, M: %.3f, G: %.3f, M/G: %.3f" % (
            corr(Nc, sp), corr(Kc, sp), corr(Mc, sp), corr(Gc, sp), corr(Mc / Gc, sp)),
        "Pearson r of the memory saving with M: %.3f, G: %.3f, M/G: %.3f" % (corr(Mc, mem), corr(Gc, mem), corr(Mc / Gc, mem)),
    ]
    for G in Gs:
        for M in Ms:
            sel = (Gc == G) & (Mc == M)
            if sel.any():
                lines.append(f"G={G:2d} M={M:5d}: speed-up {sp[sel].mean():.3f} (with unpad {spu[sel].mean():.3f}), "
                             f"memory saved {mem[sel].mean():.3f}, TFLOP/s {tf[sel].mean():.0f}")
    text = "\n".join(lines)
    print(text, file=sys.stderr)
    if args.summary:
        with open(args.summary, "w") as f:
            f.write(text + "\n")
    if args.out:
        sink.close()


if __name__ == "__main__":
    main()
