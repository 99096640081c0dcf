"""Host-side checks of the seeded input generators (no GPU)."""
import numpy as np
import torch

from workloads import CONFIGS, group_sizes, make_problem, paper_group_sizes, quantize_a, quantize_b


def test_group_size_laws():
    s = group_sizes(CONFIGS["tiny"])
    assert s.shape == (4,) and 0 in s and 1 in s and s.max() <= 300
    for name in ("gate_up", "down", "many_small", "decode"):
        cfg = CONFIGS[name]
        s = group_sizes(cfg)
        assert s.shape == (cfg.G,) and s.sum() == cfg.M_total and s.min() >= 0
        assert np.array_equal(s, group_sizes(cfg))             # reproducible
    assert (group_sizes(CONFIGS["gate_up"]) % 128 != 0).sum() >= 6
    d = group_sizes(CONFIGS["down"])
    assert d.max() > 8 * np.median(d)                          # skewed
    m = group_sizes(CONFIGS["many_small"])
    assert abs(m.mean() - 128) < 1e-9 and (m % 128 != 0).mean() > 0.9
    k = group_sizes(CONFIGS["decode"])
    assert (k < 32).sum() >= 32 and (k == 0).sum() >= 4


def test_paper_generator_sums_to_M():
    rng = np.random.default_rng(0)
    for M, G in [(8192, 32), (65536, 4), (8192, 8)]:
        v = paper_group_sizes(M, G, rng)
        assert v.sum() == M and v.min() >= 0 and v.shape == (G,)


def test_quantiser_scales_and_range():
    g = torch.Generator().manual_seed(0)
    x = torch.randn((5, 256), generator=g)
    x[1, :128] = 0
    q, s = quantize_a(x.clone())
    assert q.dtype == torch.uint8 and s.shape == (5, 2)
    assert s[1, 0] == 1.0 and not q[1, :128].any()
    deq = q.view(torch.float8_e4m3fn).float().view(5, 2, 128) * s[:, :, None]
    assert (deq.view(5, 256) - x).abs().max() <= x.abs().max() / 16 + 1e-6   # 3 mantissa bits
    assert q.view(torch.float8_e4m3fn).float().abs().max() == 448.0
    w = torch.randn((256, 384), generator=g) * 0.02
    qb, sb = quantize_b(w.clone())
    assert sb.shape == (2, 3) and qb.shape == (256, 384)
    assert not torch.isnan(qb.view(torch.float8_e4m3fn).float()).any()


def test_make_problem_tiny_is_reproducible():
    p1 = make_problem(CONFIGS["tiny"])
    p2 = make_problem(CONFIGS["tiny"])
    assert torch.equal(p1["A"], p2["A"]) and torch.equal(p1["B"], p2["B"])
    assert p1["group_offsets"].dtype == torch.int32 and p1["group_offsets"][-1] == p1["M_total"]
    assert p1["A"].shape == (p1["M_total"], 256) and p1["SB"].shape == (4, 2, 2)
