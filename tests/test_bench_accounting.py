"""The benchmark's work accounting against figures computed by hand from the layer shapes: what
`roofline.achieved` and `conv_tflops` divide by must be the method's algorithmic work, no more."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import workloads as WL  # noqa: E402


def test_call_flops_of_the_measured_configurations():
    # forward 2 M (c1 9 c_in + c2 9 c1 + C c2), backward without the first layer's data-gradient,
    # k + 1 forwards and k backwards per call
    for name, gflop in (("tiny", 0.4191), ("720p", 252.3), ("1080p", 567.7), ("batch4", 6162.6)):
        assert bench.call_flops(WL.WORKLOADS[name]) / 1e9 == pytest.approx(gflop, rel=2e-3), name
    wl = WL.WORKLOADS["720p"]
    M = 90 * 160
    fwd = 2 * M * (128 * 9 * 256 + 128 * 9 * 128 + 19 * 128)
    bwd = 2 * M * (128 * 9 * 256 + 2 * 128 * 9 * 128 + 2 * 19 * 128)
    assert bench.call_flops(wl) == 9 * fwd + 8 * bwd


def test_kernel_work_per_launch():
    wl = WL.WORKLOADS["720p"]
    w = bench.kernel_work(wl)
    M, P, C = 14400, 921600, 19
    assert w["conv12_wgrad"] == ("mfma", 2.0 * M * 128 * (2304 + 1152))          # 12.74 GFLOP
    assert w["conv12_wgrad"][1] / 1e9 == pytest.approx(12.740, abs=1e-3)
    assert w["conv1_fwd"][1] / 1e9 == pytest.approx(8.4935, abs=1e-3)
    assert w["conv2_dgrad"][1] / 1e9 == pytest.approx(4.2467, abs=1e-3)
    assert w["upsample_ce_grad"] == ("alu", 19.0 * C * P)
    assert w["sgd_update"] == ("hbm", 14.0 * 445075)
    assert bench.kernel_work(WL.WORKLOADS["1080p"])["sgd_update"] == ("hbm", 22.0 * 445075)     # momentum


def test_peaks_are_the_published_ones():
    assert bench.PEAK_TFLOPS_BF16 == 2500.0 and bench.PEAK_TFLOPS_F32 == 157.3 and bench.PEAK_HBM_GBS == 8000.0


def test_traffic_figures_belong_to_the_sources_as_they_stand():
    """Every (workload, kernel) entry of the measured-traffic table must match the kernel source in
    the tree, or the bench line would carry `traffic: null` for it."""
    stale = [k for k in bench.MEASURED_TRAFFIC if bench.measured_traffic(k[1], k[0]) is None]
    assert not stale, f"re-measure FETCH_SIZE / WRITE_SIZE for {stale} and refresh profiles/"
    for wl in ("720p", "1080p", "batch4"):
        assert (wl, "conv12_wgrad_mfma") in bench.MEASURED_TRAFFIC and (wl, "upsample_ce_grad") in bench.MEASURED_TRAFFIC
