"""The library's calls inside a HIP graph: it allocates nothing, synchronises nothing and keeps no state, so a chain
of its launches can be captured once and replayed (the launch-bound case: many small expert GEMMs per layer).
Every replay is checked against the eager result, with eager work and synchronisations between the replays and
with new contents in the input buffer."""
import numpy as np
import pytest
import torch

import paper_2508_16584_amd as gg
from workloads.quantize import quantize_b

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_captured_chain_replays_equal_eager():
    sizes = np.array([130, 0, 257, 64, 1])
    G, M, K, inter = len(sizes), int(sizes.sum()), 1024, 256
    N = 2 * inter
    gen = torch.Generator(device=DEV)
    gen.manual_seed(8100)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)).to(DEV)
    src = torch.randperm(M, generator=gen, device=DEV).to(torch.int32)
    B1 = torch.empty((G, N, K), dtype=torch.uint8, device=DEV)
    SB1 = torch.empty((G, N // 128, K // 128), dtype=torch.float32, device=DEV)
    B2 = torch.empty((G, K, inter), dtype=torch.uint8, device=DEV)
    SB2 = torch.empty((G, K // 128, inter // 128), dtype=torch.float32, device=DEV)
    for g in range(G):
        B1[g], SB1[g] = quantize_b(torch.randn((N, K), generator=gen, device=DEV) * 0.05)
        B2[g], SB2[g] = quantize_b(torch.randn((K, inter), generator=gen, device=DEV) * 0.05)
    xs = [torch.randn((M, K), generator=gen, device=DEV).to(torch.bfloat16) for _ in range(3)]
    X = xs[0].clone()
    buf = dict(
        A1=torch.empty((M, K), dtype=torch.uint8, device=DEV), SA1=torch.empty((K // 128, M), dtype=torch.float32, device=DEV),
        H=torch.empty((M, N), dtype=torch.bfloat16, device=DEV),
        A2=torch.empty((M, inter), dtype=torch.uint8, device=DEV), SA2=torch.empty((inter // 128, M), dtype=torch.float32, device=DEV),
        Y=torch.empty((M, K), dtype=torch.bfloat16, device=DEV),
        A2f=torch.empty((M, inter), dtype=torch.uint8, device=DEV), SA2f=torch.empty((inter // 128, M), dtype=torch.float32, device=DEV),
        Yf=torch.empty((M, K), dtype=torch.bfloat16, device=DEV))

    def chain():
        gg.quantize_rows(X, src, A=buf["A1"], SA=buf["SA1"], sa_kmajor=True)
        gg.grouped_gemm(buf["A1"], buf["SA1"], B1, SB1, off, C=buf["H"], sa_kmajor=True)
        gg.swiglu_quantize_rows(buf["H"], A=buf["A2"], SA=buf["SA2"], sa_kmajor=True)
        gg.grouped_gemm(buf["A2"], buf["SA2"], B2, SB2, off, C=buf["Y"], sa_kmajor=True)
        # the same with the activation in the first GEMM's epilogue
        gg.grouped_gemm_swiglu(buf["A1"], buf["SA1"], B1, SB1, off, A2=buf["A2f"], SA2=buf["SA2f"], sa_kmajor=True)
        gg.grouped_gemm(buf["A2f"], buf["SA2f"], B2, SB2, off, C=buf["Yf"], sa_kmajor=True)

    # eager references for the three inputs (this also does the one-time set-up of every kernel outside the capture)
    want = []
    for x in xs:
        X.copy_(x)
        chain()
        torch.cuda.synchronize()
        want.append({k: v.clone() for k, v in buf.items()})
        assert torch.equal(buf["Y"].view(torch.int16), buf["Yf"].view(torch.int16))

    graph = torch.cuda.CUDAGraph()
    X.copy_(xs[0])
    with torch.cuda.graph(graph):
        chain()
    for rep, which in enumerate([0, 1, 2, 1]):
        X.copy_(xs[which])
        for v in buf.values():                                # eager work between the replays: wipe every output
            v.view(torch.uint8).fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in buf.items():
            assert torch.equal(v.view(torch.uint8), want[which][k].view(torch.uint8)), f"replay {rep}: {k} differs from the eager run"
