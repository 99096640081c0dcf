"""Real-valued draws -> e4m3 bytes + float32 block scales (input side only).

Per (row, 128-wide K block) of A and per 128x128 block of every B^g:
scale = amax / 448, byte = round-to-nearest-even e4m3 of x / scale (saturating
at +-448); an all-zero block gets scale 1.  Scales are dequantisation
multipliers.  The conversion itself is torch's float8_e4m3fn cast; whatever it
produces, the oracle and the HIP library read the same bytes, so quantiser
details never enter a parity comparison.
"""
from __future__ import annotations

import numpy as np
import torch

from .configs import WorkloadConfig, group_sizes

E4M3_MAX = 448.0
BLK = 128


def _to_e4m3_bytes(x: torch.Tensor) -> torch.Tensor:
    return x.clamp_(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn).view(torch.uint8)


def quantize_a(x: torch.Tensor):
    """x float32 [M, K], K % 128 == 0  ->  (uint8 [M, K], float32 [M, K/128])."""
    M, K = x.shape
    assert K % BLK == 0
    xb = x.view(M, K // BLK, BLK)
    amax = xb.abs().amax(dim=2)
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax))
    q = _to_e4m3_bytes(xb / scale[:, :, None]).view(M, K)
    return q.contiguous(), scale.contiguous()


def quantize_b(w: torch.Tensor):
    """w float32 [N, K], both % 128 == 0  ->  (uint8 [N, K], float32 [N/128, K/128])."""
    N, K = w.shape
    assert N % BLK == 0 and K % BLK == 0
    wb = w.view(N // BLK, BLK, K // BLK, BLK)
    amax = wb.abs().amax(dim=(1, 3))
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax))
    q = _to_e4m3_bytes(wb / scale[:, None, :, None]).view(N, K)
    return q.contiguous(), scale.contiguous()


def make_problem(cfg: WorkloadConfig, device="cpu", seed: int | None = None,
                 sizes: np.ndarray | None = None, a_std=1.0, b_std=0.02):
    """Draw one problem instance of a config.

    Returns a dict of torch tensors on `device`:
      A uint8 [M_total, K], SA float32 [M_total, K/128], B uint8 [G, N, K],
      SB float32 [G, N/128, K/128], group_offsets int32 [G+1], plus "sizes"
      (NumPy int64[G]) and the scalars G, M_total, N, K.
    A ~ N(0, a_std^2), B^g ~ N(0, b_std^2), drawn group by group so that the
    largest config never holds more than one group in float32.
    """
    seed = cfg.seed if seed is None else seed
    if sizes is None:
        sizes = group_sizes(cfg, seed)
    sizes = np.asarray(sizes, dtype=np.int64)
    G, K, N = sizes.shape[0], cfg.K, cfg.N
    M_total = int(sizes.sum())
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    A = torch.empty((M_total, K), dtype=torch.uint8, device=dev)
    SA = torch.empty((M_total, K // BLK), dtype=torch.float32, device=dev)
    chunk = 4096
    for r0 in range(0, M_total, chunk):
        r1 = min(M_total, r0 + chunk)
        x = torch.randn((r1 - r0, K), generator=gen, device=dev, dtype=torch.float32) * a_std
        A[r0:r1], SA[r0:r1] = quantize_a(x)
    B = torch.empty((G, N, K), dtype=torch.uint8, device=dev)
    SB = torch.empty((G, N // BLK, K // BLK), dtype=torch.float32, device=dev)
    for g in range(G):
        w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * b_std
        B[g], SB[g] = quantize_b(w)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    return {
        "A": A, "SA": SA, "B": B, "SB": SB,
        "group_offsets": torch.from_numpy(off).to(dev),
        "sizes": sizes, "G": G, "M_total": M_total, "N": N, "K": K,
    }
