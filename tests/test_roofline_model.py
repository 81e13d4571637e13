"""The throughput model restated from the paper reproduces every printed entry of Table 2."""
import os

import numpy as np

from paper_2408_11200_amd import roofline


def test_table2_arithmetic(golden_dir):
    rows = [[float(t) for t in l.split()] for l in open(os.path.join(golden_dir, "table2_sol.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    for G, t_meas, sol_best, sol_worst, t_c, t_mb, t_mw in rows:
        m = roofline.paper_sol(N=2 ** 17, d_in=32, d_out=32, K=4, G=int(G), p_flop=38.7e12, p_bw=768e9)
        assert abs(m["t_compute"] * 1e3 - t_c) < 5e-5
        assert abs(m["t_mem_best"] * 1e3 - t_mb) < 5e-5 + 1e-4     # printed to 4 decimals
        assert abs(m["t_mem_worst"] * 1e3 - t_mw) < 5e-5
        assert abs(m["t_sol_best"] * 1e3 - sol_best) < 5e-5
        assert abs(m["t_sol_worst"] * 1e3 - sol_worst) < 5e-5


def test_mi355x_model_for_the_headline_layer():
    e = roofline.edge_evals(16384, 512, 512)
    assert e == 4294967296
    assert roofline.algorithmic_flops_per_edge(4) == 30
    b = roofline.algorithmic_hbm_bytes(16384, 512, 512, 20, 3)
    assert abs(b - 246e6) < 1e6
    t_valu = e * 30 / roofline.MI355X_FP32_VECTOR_FLOPS
    assert abs(t_valu - 819e-6) < 1e-6


def test_bench_reads_its_traffic_figure_from_the_tracked_profile():
    """bench.py takes roofline.traffic from a machine-readable line of the tracked rocprofv3 summary: the line must
    parse, name the commit it was measured at, and only answer for the workload and kernel families it covers."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    total, src = bench.measured_traffic("c3", "backward_walk")
    assert src["file"] == bench.TRAFFIC_FILE and len(src["source_commit"]) >= 7
    assert total == src["read"] + src["written"] and 1e9 < total < 4e9
    fwd, _ = bench.measured_traffic("c3", "forward_pairs")
    assert 1e8 < fwd < 1e9
    assert bench.measured_traffic("c3", "forward_lds") == (None, None)       # a kernel family the summary does not cover
    assert bench.measured_traffic("c4", "backward_walk") == (None, None)     # another workload
    assert set(bench.KERNEL_ROLE.values()) <= set(bench.ROLE_SHARE)
