"""The flop/byte counter reproduces the value the paper prints (Appendix B) and the ridge (Appendix A)."""

import os

from paper_2511_07399_amd import cost_model as cm
from paper_2511_07399_amd import workloads as wk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "appendix_b_intensity.txt")


def read_golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_paper_intensity_worked_example():
    g = read_golden()
    got = cm.paper_intensity(int(g["C"]), int(g["L_q"]), int(g["L_kv"]), int(g["N"]), int(g["b"]),
                             gamma=g["gamma_GiB"] * cm.GIB, peak_flops=g["peak_TFLOPS"] * 1e12,
                             bandwidth=g["bandwidth_TBps"] * 1e12)
    assert round(got, 2) == g["intensity_printed"]
    assert g["peak_TFLOPS"] * 1e12 / (g["bandwidth_TBps"] * 1e12) == g["ridge_printed"]
    # without the roll/concat copies the same model is compute-bound even on the paper's GPU
    assert cm.paper_intensity(2048, 1536, 9216, 30) > 1.0


def test_paper_flops_terms():
    # 24 b L C^2 = QKV (3) + out (1) + FFN with F = 4C (8) matrix products of 2 L C^2 flops each
    assert cm.paper_flops(64, 10, 0, 1) == 12 * 2 * 10 * 64 * 64
    assert cm.paper_flops(64, 10, 30, 1) - cm.paper_flops(64, 10, 0, 1) == cm.attention_flops(10, 30, 64)
    assert cm.paper_flops(64, 10, 30, 3, b=2) == 6 * cm.paper_flops(64, 10, 30, 1)


def test_block_counts_for_named_workloads():
    wl = wk.WORKLOADS["wan1.3b-block"]
    f = cm.block_flops(wl.B * wl.L, wl.C, wl.F, wl.S + wl.W, wl.L_t)
    assert f == wl.block_flops()
    assert abs(f / 1e9 - 107.9) < 0.1
    wl = wk.WORKLOADS["wan14b-step"]
    assert abs(wl.block_flops() / 1e9 - 687.2) < 0.2
    wl = wk.WORKLOADS["wan14b-480p-b4"]
    assert wl.L == 4680 and wl.S + wl.W == 10920
    assert abs(wl.block_flops() / 1e12 - 15.57) < 0.02
