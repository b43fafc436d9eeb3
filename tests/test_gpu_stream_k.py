"""GPU parity of the stream-K tail (tiles that do not fill a whole number of rounds on the compute units: with a
workspace the k range of the left-over tiles is shared out over all workgroups and pieces are added by the tile's owner).

Gate and derived bound as in the other parity tests.  The pieces of a tile are added in a fixed order, so a run with a
workspace is bitwise reproducible; it is not bitwise equal to the run without one (another summation order in fp32)."""
import numpy as np
import pytest
import torch

from oracle import codec, tp_gemm
from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu

GATE = {"bf16": 1e-2, "fp8": 5e-2}
U32 = 2.0 ** -24


def gate_err(gpu, ref):
    return float(np.max(np.abs(gpu - ref) / (np.abs(ref) + 1.0)))


def check_ag(P, rank, dtype, inp, res, K):
    A = tp_gemm.gather_chunks(inp["chunks"])
    ref = tp_gemm.ag_gemm(P, rank, A, inp["B_local"], dtype, inp["scale_a"], inp["scale_b"])
    mag = tp_gemm.abs_product(A, inp["B_local"], dtype, inp["scale_a"], inp["scale_b"])
    assert res["status"][0] == 0, res["status"]
    got = codec.bf16_decode(res["C_bits"])
    assert not np.isnan(got).any()
    assert gate_err(got, ref["C"]) <= GATE[dtype]
    bound = 2 * K * U32 * mag + 2.0 ** -8 * np.abs(ref["C"]) + 2.0 ** -133
    assert np.all(np.abs(got - ref["C"]) <= bound)


# 288 tiles of 256 x 256 (18 x 16): on g workgroups that is whole rounds plus a tail of 288 mod g tiles
@pytest.mark.parametrize("dtype,K", [("bf16", 1024), ("fp8", 2048)])
@pytest.mark.parametrize("comm_cus", [0, 64, 192])
def test_ag_gemm_with_a_workspace(dtype, K, comm_cus):
    P, rank, M, N = 2, 1, 4608, 8192
    inp = wl.ag_gemm_inputs(P, M, N, K, dtype, rank, seed=31)
    kw = dict(scale_a=inp["scale_a"], scale_b=inp["scale_b"], comm_cus=comm_cus)
    res = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], workspace=True, **kw)
    check_ag(P, rank, dtype, inp, res, K)
    again = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], workspace=True, epoch=7, **kw)
    assert np.array_equal(again["C_bits"], res["C_bits"])          # fixed piece order: bitwise reproducible
    if comm_cus == 0:
        plain = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], **kw)
        check_ag(P, rank, dtype, inp, plain, K)


def test_ag_gemm_workspace_reused_across_epochs_and_arrival_orders():
    """One workspace, zeroed once, serves calls with growing epochs; chunks arriving live in any order give the same bits."""
    P, rank, M, N, K = 4, 2, 4608, 4 * 4096, 1024
    inp = wl.ag_gemm_inputs(P, M, N, K, "bf16", rank, seed=32)
    plan = pk.pk_ag_gemm_plan(P, M, N, K, "bf16")
    ws = torch.zeros(plan.workspace_bytes // 4, dtype=torch.int32, device="cuda")
    base = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], workspace=ws, epoch=1)
    check_ag(P, rank, "bf16", inp, base, K)
    peers = [q for q in range(P) if q != rank]
    for i, order in enumerate([peers, peers[::-1], [peers[1], peers[0], peers[2]]]):
        res = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], workspace=ws, epoch=2 + i,
                             deliver="emu", order=order, gap_us=(0, 50, 10)[i], fetch_A=False)
        assert res["status"][0] == 0
        assert np.array_equal(res["C_bits"], base["C_bits"]), f"order {order}"


def test_ag_gemm_small_tiles_with_a_workspace():
    """288 tiles of 128 x 128 (a problem too small for the large tiles), 16 k-tiles each."""
    P, rank, M, N, K = 1, 0, 2304, 2048, 1024
    inp = wl.ag_gemm_inputs(P, M, N, K, "bf16", rank, seed=33)
    assert pk.pk_ag_gemm_plan(P, M, N, K, "bf16").tile_m == 128
    res = hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"], workspace=True)
    check_ag(P, rank, "bf16", inp, res, K)


@pytest.mark.parametrize("comm_cus", [0, 192])
def test_gemm_rs_with_a_workspace(comm_cus):
    P, rank, M, N, K = 2, 0, 4608, 4096, 2048
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=34)
    res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], workspace=True,
                         comm_cus=comm_cus)
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], "bf16", inp["partials"])
    assert res["status"][0] == 0, res["status"]
    got = codec.bf16_decode(res["out_bits"])
    assert gate_err(got, ref["out"]) <= GATE["bf16"]
    mp = M // P
    for q in range(P):
        if q != rank:
            assert gate_err(res["outgoing"][q], ref["own"][q * mp:(q + 1) * mp]) <= 1e-5
    assert np.all(res["flags_out"][1 - rank] == 1) and np.all(res["flags_in"][rank] == 1)


def test_workspace_too_small_is_rejected():
    P, rank, M, N, K = 2, 1, 4608, 8192, 1024
    inp = wl.ag_gemm_inputs(P, M, N, K, "bf16", rank, seed=35)
    with pytest.raises(pk.PkError) as e:
        hz.run_ag_gemm(P, rank, M, N, K, "bf16", inp["chunks"], inp["B_local"],
                       workspace=torch.zeros(1024 + 65536, dtype=torch.int32, device="cuda"))
    assert e.value.code == pk.ERR_ARG
