"""The seeded generators: determinism, shapes, distributions and the exact representability of what they emit."""
import numpy as np

from oracle import codec
from paper_2511_13940_amd import workloads as wl


def test_configs_match_the_stated_local_shapes():
    assert wl.CONFIGS["cfg1"].local_mnk == (256, 256, 256)
    assert wl.CONFIGS["cfg2"].local_mnk == (2048, 1024, 2048)
    assert wl.CONFIGS["cfg3"].local_mnk == (8192, 8192, 3584)
    assert wl.CONFIGS["cfg4"].local_mnk == (8192, 3584, 8192)
    assert wl.CONFIGS["cfg5"].local_mnk == (16384, 16384, 2048)
    assert wl.CONFIGS["cfg3"].flops == 2 * 8192 * 8192 * 3584


def test_gemm_rs_inputs_seeded_and_distributed():
    c = wl.CONFIGS["cfg1"]
    a = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, rank=0, seed=1)
    b = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, rank=0, seed=1)
    d = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, rank=1, seed=1)
    assert np.array_equal(a["A_local"], b["A_local"]) and np.array_equal(a["partials"], b["partials"])
    assert not np.array_equal(a["A_local"], d["A_local"])
    assert a["A_local"].shape == (256, 256) and a["A_local"].dtype == np.uint16
    assert a["B_local"].shape == (256, 256)
    assert a["partials"].shape == (2, 128, 256) and a["partials"].dtype == np.float32
    assert not a["partials"][0].any() and a["partials"][1].any()
    x = codec.bf16_decode(a["A_local"])
    assert abs(x.std() * np.sqrt(c.K) - 1.0) < 0.02 and abs(x.mean()) < 1e-3
    sig_p = np.sqrt(c.K // c.P) / c.K
    assert abs(a["partials"][1].std() / sig_p - 1.0) < 0.02


def test_fp8_inputs_scale_and_range():
    inp = wl.gemm_rs_inputs(2, 64, 64, 128, "fp8", rank=0, seed=2)
    assert inp["A_local"].dtype == np.uint8 and inp["scale_a"].dtype == np.float32
    v = codec.e4m3_decode(inp["A_local"])
    assert np.all(np.isfinite(v)) and np.max(np.abs(v)) == 448.0
    # dequantised values keep the input distribution (std 1/sqrt(K)) to within quantisation noise
    assert abs((v * float(inp["scale_a"])).std() * np.sqrt(128) - 1.0) < 0.05


def test_arrival_orders():
    assert wl.arrival_order(8, 3, "ring") == [4, 5, 6, 7, 0, 1, 2]
    r = wl.arrival_order(4, 1, "random", seed=5)
    assert sorted(r) == [0, 2, 3] and r == wl.arrival_order(4, 1, "random", seed=5)


def test_global_problem_slices():
    g = wl.global_problem(8, 12, 16, "bf16", seed=1)
    a1, b1 = wl.slice_gemm_rs(g, 4, 1)
    assert np.array_equal(a1, g["A"][:, 4:8]) and np.array_equal(b1, g["B"][4:8, :])
    c2, b2 = wl.slice_ag_gemm(g, 4, 2)
    assert np.array_equal(c2, g["A"][4:6]) and np.array_equal(b2, g["B"][:, 6:9])


def test_ag_inputs():
    inp = wl.ag_gemm_inputs(4, 16, 32, 24, "bf16", rank=2, seed=0, order="ring")
    assert len(inp["chunks"]) == 4 and inp["chunks"][0].shape == (4, 24)
    assert inp["B_local"].shape == (24, 8) and inp["order"] == [3, 0, 1]
    f = wl.ag_gemm_inputs(2, 8, 32, 16, "fp8", rank=0)
    assert f["chunks"][1].dtype == np.uint8 and f["scale_a"] is not None
