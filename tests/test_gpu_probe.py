"""The measurement probes of include/gg_probe.h run and report figures of the right order (short runs: these are
not the measurements themselves, `python bench.py --op ceilings` makes those)."""
import pytest

import paper_2508_16584_amd as gg

pytestmark = pytest.mark.gpu


def test_matrix_loops_report_plausible_rates():
    rates = [gg.probe_mfma(mode, 1, 2000) for mode in range(4)]
    # between a tenth of the FP8 dense peak and the peak itself (5.0 PFLOP/s)
    assert all(500.0 < r < 5100.0 for r in rates), rates
    # the scale fusion (mode 1) cannot be faster than the bare accumulating loop (mode 0) by more than noise
    assert rates[1] < 1.05 * rates[0]


def test_issue_mix_loops_run_and_more_instructions_are_not_faster():
    base = gg.probe_issue_mix(0, 0, 0, 2000)
    heavy = gg.probe_issue_mix(2, 1, 2, 2000)
    assert 500.0 < heavy < 1.05 * base < 5400.0, (base, heavy)


def test_hbm_and_fetch_streams_report_plausible_rates():
    read = gg.probe_hbm(0, 512 << 20, 2)
    copy = gg.probe_hbm(1, 512 << 20, 2)
    assert 1000.0 < read < 8100.0 and 1000.0 < copy < 8100.0, (read, copy)
    for pattern in range(3):
        gbps, per_clk_cu = gg.probe_lds_fetch(pattern, 3, 2)
        assert 1000.0 < gbps < 60000.0 and 1.0 < per_clk_cu < 128.0, (pattern, gbps, per_clk_cu)


def test_kernels_with_parts_left_out_run_and_leaving_out_is_not_slower():
    """The measurement builds of the second GEMM kernel and of the weight-gradient kernel on small problems: they
    run, and a build with its fetches and stores left out is not slower than the kernel as launched."""
    full = gg.probe_gemm_kstep(192, 0, 4, 768, 1024, 2048, 3)
    bare = gg.probe_gemm_kstep(192, 13, 4, 768, 1024, 2048, 3)
    assert 1.0 < bare < 1.05 * full < 5000.0, (full, bare)
    full = gg.probe_wgrad_parts(0, 4, 500, 1024, 1024, 3)
    bare = gg.probe_wgrad_parts(3, 4, 500, 1024, 1024, 3)
    alone = gg.probe_wgrad_parts(31, 4, 500, 1024, 1024, 3)
    assert 1.0 < alone < 1.05 * bare < 1.1 * full < 5000.0, (full, bare, alone)
