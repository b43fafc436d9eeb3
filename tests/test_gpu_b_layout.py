"""GPU parity of the k-contiguous layout of the second operand (PK_B_K_CONTIGUOUS: the N x K transpose of B is passed).
The oracle is called on the matrix itself (the transposed bits transposed back); the fragments that reach the matrix cores
and their order are the same as on the row-major path, so the two GPU results must also be bit-identical."""
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


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 704, 400, 512, 1),                    # small tiles, ragged rows and columns
    (4, 4 * 136, 1040, 1024, 2),               # shard smaller than two tiles
    (2, 4608, 4096, 512, 0),                   # 288 large tiles, one of the tile rows ragged
])
def test_gemm_rs_k_contiguous_b(dtype, P, M, N, K, rank):
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=61)
    Bt = np.ascontiguousarray(np.asarray(inp["B_local"]).T)
    kw = dict(scale_a=inp.get("scale_a"), scale_b=inp.get("scale_b"))
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], Bt, inp["partials"], b_layout="nk", **kw)
    assert res["status"][0] == 0, res["status"]
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], np.ascontiguousarray(Bt.T), dtype, inp["partials"], **kw)
    got = codec.bf16_decode(res["out_bits"])
    assert gate_err(got, ref["out"]) <= GATE[dtype]
    mag = tp_gemm.abs_product(inp["A_local"], np.ascontiguousarray(Bt.T), dtype, **kw)
    mp = M // P
    for q in range(P):
        slot = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        assert np.all(np.abs(slot - ref["outgoing"][q]) <= 2 * (K // P) * U32 * mag[q * mp:(q + 1) * mp] + 1e-30)
    plain = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], **kw)
    assert np.array_equal(res["out_bits"], plain["out_bits"])
    for q in range(P):
        if q != rank:
            assert np.array_equal(res["outgoing"][q], plain["outgoing"][q])


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (4, 384, 1088, 384, 3),
    (2, 4608, 8192, 512, 1),
])
def test_ag_gemm_k_contiguous_b(dtype, P, M, N, K, rank):
    if dtype == "fp8" and K % 128:
        pytest.skip("shape not valid for fp8")
    inp = wl.ag_gemm_inputs(P, M, N, K, dtype, rank, seed=62)
    Bt = np.ascontiguousarray(np.asarray(inp["B_local"]).T)
    kw = dict(scale_a=inp["scale_a"], scale_b=inp["scale_b"])
    res = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], Bt, b_layout="nk", fetch_A=False, **kw)
    assert res["status"][0] == 0, res["status"]
    A = tp_gemm.gather_chunks(inp["chunks"])
    ref = tp_gemm.ag_gemm(P, rank, A, np.ascontiguousarray(Bt.T), dtype, inp["scale_a"], inp["scale_b"])
    got = codec.bf16_decode(res["C_bits"])
    assert gate_err(got, ref["C"]) <= GATE[dtype]
    mag = tp_gemm.abs_product(A, np.ascontiguousarray(Bt.T), dtype, inp["scale_a"], inp["scale_b"])
    assert np.all(np.abs(got - ref["C"]) <= 2 * K * U32 * mag + 2.0 ** -8 * np.abs(ref["C"]) + 2.0 ** -133)
    plain = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], fetch_A=False, **kw)
    assert np.array_equal(res["C_bits"], plain["C_bits"])


def test_k_contiguous_b_live_arrival_and_workspace():
    """The layout composes with live chunk arrival; a workspace is accepted (the stream-K tail is built for the row-major
    layout only, so the tiles stay whole and the result equals the plain one)."""
    P, rank, M, N, K = 2, 1, 4608, 8192, 1024
    inp = wl.ag_gemm_inputs(P, M, N, K, "bf16", rank, seed=63)
    Bt = np.ascontiguousarray(np.asarray(inp["B_local"]).T)
    base = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], Bt, b_layout="nk", workspace=True, fetch_A=False)
    live = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], Bt, b_layout="nk", workspace=True, fetch_A=False,
                          deliver="emu", epoch=5)
    assert base["status"][0] == 0 and live["status"][0] == 0
    assert np.array_equal(base["C_bits"], live["C_bits"])
    plain = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], fetch_A=False)
    assert np.array_equal(base["C_bits"], plain["C_bits"])
