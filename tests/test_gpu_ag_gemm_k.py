"""GPU parity of pk_ag_gemm_k (all-gather along the last dimension of A + GEMM) against the float64 oracle, through the
C ABI.  Gates and derived bound as for pk_ag_gemm."""
import itertools

import numpy as np
import pytest

from oracle import codec, tp_gemm
from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu

GATE = {"bf16": 1e-2, "fp8": 5e-2}
U32 = 2.0 ** -24


def gate_err(gpu, ref):
    return float(np.max(np.abs(gpu - ref) / (np.abs(ref) + 1.0)))


def inputs(P, M, N, K, dtype, rank, seed):
    """A (M x K) cut into P column chunks, B_local = B[:, N_rank]."""
    g = wl.global_problem(M, N, K, dtype, seed=seed)
    kp, ns = K // P, N // P
    chunks = [np.ascontiguousarray(g["A"][:, q * kp:(q + 1) * kp]) for q in range(P)]
    return {"chunks": chunks, "B_local": np.ascontiguousarray(g["B"][:, rank * ns:(rank + 1) * ns]),
            "scale_a": g["scale_a"], "scale_b": g["scale_b"]}


def check(P, rank, dtype, inp, res, K, act="none"):
    A = tp_gemm.gather_kchunks(inp["chunks"])
    ref = tp_gemm.activation(tp_gemm.local_product(A, inp["B_local"], dtype, inp["scale_a"], inp["scale_b"]), act)
    mag = tp_gemm.abs_product(A, inp["B_local"], dtype, inp["scale_a"], inp["scale_b"])
    assert res["status"][0] == 0, res["status"]
    got = codec.bf16_decode(res["C_bits"])
    assert not np.isnan(got).any()
    assert gate_err(got, ref) <= GATE[dtype]
    bound = 1.13 * 2 * K * U32 * mag + 2.0 ** -8 * np.abs(ref) + 16 * U32 * (np.abs(ref) + 1.0) + 2.0 ** -133
    assert np.all(np.abs(got - ref) <= bound)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 256, 2 * 256, 2 * 128, 0),
    (4, 200, 4 * 264, 4 * 128, 3),       # ragged rows (M not a multiple of P or of the tile) and columns
    (1, 256, 256, 256, 0),               # P = 1: plain GEMM
    (3, 130, 3 * 16, 3 * 256, 1),        # odd P, several k-tiles per chunk
    (8, 128, 8 * 32, 8 * 128, 5),        # chunk = one or two k-tiles: shorter than the load pipeline
])
def test_small_tiles(dtype, P, M, N, K, rank):
    if dtype == "fp8" and (N // P) % 16:
        pytest.skip("shape not valid for fp8")
    inp = inputs(P, M, N, K, dtype, rank, seed=23)
    res = hz.run_ag_gemm_k(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], inp["scale_a"], inp["scale_b"], epoch=2)
    check(P, rank, dtype, inp, res, K)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_big_tiles_with_activation(dtype):
    P, rank, M, N, K = 2, 1, 4096 - 24, 2 * (4096 - 48), 2 * 256
    assert pk.pk_ag_gemm_k_plan(P, M, N, K, dtype).tile_m == 256
    inp = inputs(P, M, N, K, dtype, rank, seed=24)
    res = hz.run_ag_gemm_k(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], inp["scale_a"], inp["scale_b"], act="silu")
    check(P, rank, dtype, inp, res, K, act="silu")


def test_all_arrival_orders_bitwise_identical_and_no_early_reads():
    """All 6 orders of the 3 peer chunks, delivered by strided copies into NaN-poisoned columns while the GEMM runs."""
    P, rank, M, N, K = 4, 2, 1024, 4 * 512, 4 * 512
    inp = inputs(P, M, N, K, "bf16", rank, seed=25)
    base = hz.run_ag_gemm_k(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"])
    check(P, rank, "bf16", inp, base, K)
    full = tp_gemm.gather_kchunks(inp["chunks"])
    peers = [q for q in range(P) if q != rank]
    for i, order in enumerate(itertools.permutations(peers)):
        res = hz.run_ag_gemm_k(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], deliver="dma", order=list(order),
                               epoch=i + 1)
        assert res["status"][0] == 0
        assert np.array_equal(res["C_bits"], base["C_bits"]), f"order {order}"
        assert np.array_equal(res["A_after"].view(np.uint16), full)
        assert np.all(res["flags"][peers] == i + 1)


def test_column_shards_side_by_side_give_the_full_product():
    P, M, N, K = 4, 384, 4 * 128, 4 * 128
    g = wl.global_problem(M, N, K, "bf16", seed=26)
    kp, ns = K // P, N // P
    chunks = [np.ascontiguousarray(g["A"][:, q * kp:(q + 1) * kp]) for q in range(P)]
    cols = []
    for r in range(P):
        res = hz.run_ag_gemm_k(P, r, M, N, K, "bf16", chunks, np.ascontiguousarray(g["B"][:, r * ns:(r + 1) * ns]))
        assert res["status"][0] == 0
        cols.append(codec.bf16_decode(res["C_bits"]))
    full = tp_gemm.local_product(g["A"], g["B"], "bf16")
    got = np.concatenate(cols, axis=1)
    assert gate_err(got, full) <= GATE["bf16"]
    assert np.all(np.abs(got - full) <= 2 * K * U32 * tp_gemm.abs_product(g["A"], g["B"], "bf16") + 2.0 ** -8 * np.abs(full))


def test_missing_chunk_times_out_instead_of_hanging():
    P, rank, M, N, K = 4, 0, 256, 4 * 128, 4 * 128
    inp = inputs(P, M, N, K, "bf16", rank, seed=27)
    res = hz.run_ag_gemm_k(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], epoch=5, withhold=2, timeout_us=2000)
    assert res["status"][0] == pk.ERR_TIMEOUT and res["status"][1] == 2 and res["status"][2] == 1
    assert np.all(res["C_bits"] == 0xFFFF)                          # no tile was stored (every tile needs chunk 2)
