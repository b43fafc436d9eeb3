"""The cost relations against the values the paper prints (section 3.1.3, Table 3)."""
import os

from oracle import cost_model


def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_hiding_threshold_printed_value(golden_dir):
    for s, R, B, printed in _rows(os.path.join(golden_dir, "hiding_threshold.txt")):
        k = cost_model.hiding_threshold_K(float(s), float(R), float(B))
        assert int(k) == int(printed)            # 2197.8 is printed as "about 2197"
        # the threshold is where the two per-tile times cross, for any tile shape
        for m, n in [(16, 16), (128, 256), (256, 256)]:
            tc = cost_model.tile_compute_time(m, n, k, float(R))
            tm = cost_model.tile_comm_time(m, n, float(s), float(B))
            assert abs(tc - tm) <= 1e-12 * tm


def test_table3_comm_ratio(golden_dir):
    for K, t_gemm, t_fused, pct, kind in _rows(os.path.join(golden_dir, "table3_gemm_rs_ablation.txt")):
        r = 100.0 * cost_model.comm_ratio(float(t_gemm), float(t_fused))
        if kind == "eq":
            assert round(r) == int(pct), (K, r)
        else:
            assert 0.0 <= r < float(pct), (K, r)


def test_kernel_time_composition():
    assert cost_model.kernel_time(1.0, 5.0, 3.0, 4.0, 0.5, 0.25) == 1.0 + 5.0 + 0.5 + 0.25
    assert cost_model.kernel_time(0.0, 1.0, 2.0, 9.0, 0.0, 0.0) == 9.0
