"""Compute-unit partition (the paper's inter-SM overlap with an SM split): the op runs on the compute stream of a
pk_partition, the emulated peers on its communicator stream, on disjoint compute units.  Results must equal the
pre-landed runs on the default stream bit for bit, and pass the oracle gates."""
import numpy as np
import pytest
import torch

from oracle import codec
from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz
from tests.test_gpu_ag_gemm import check_ag
from tests.test_gpu_gemm_rs import check_rs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def partition():
    comp, comm = pk.pk_partition_create(32)
    assert comp and comm and comp != comm
    yield comp, comm
    torch.cuda.synchronize()
    pk.pk_partition_destroy(comp, comm)


def test_ag_gemm_on_a_partition(partition):
    c = wl.CONFIGS["cfg2"]
    rank = 2
    inp = wl.ag_gemm_inputs(c.P, c.M, c.N, c.K, c.dtype, rank, seed=5)
    base = hz.run_ag_gemm(c.P, rank, c.M, c.N, c.K, c.dtype, inp["chunks"], inp["B_local"])
    check_ag(c.P, rank, c.dtype, inp, base, c.K)
    for i, (n_wg, gap) in enumerate([(32, 0), (128, 30)]):
        res = hz.run_ag_gemm(c.P, rank, c.M, c.N, c.K, c.dtype, inp["chunks"], inp["B_local"], deliver="emu",
                             order=inp["order"], gap_us=gap, epoch=i + 1, comm_cus=32, n_wg=n_wg, partition=partition)
        assert res["status"][0] == 0
        assert np.array_equal(res["C_bits"], base["C_bits"])


def test_gemm_rs_on_a_partition_big_tiles(partition):
    P, rank, M, N, K = 4, 3, 4096, 4096, 4 * 256
    assert pk.pk_gemm_rs_plan(P, M, N, K, "bf16").tile_m == 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=21)
    base = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"])
    check_rs(P, rank, "bf16", inp, base, K // P)
    for i, n_wg in enumerate([32, 128]):
        order = wl.arrival_order(P, rank, "random", seed=i)
        res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], deliver="emu",
                             order=order, epoch=i + 1, comm_cus=32, n_wg=n_wg, partition=partition)
        assert res["status"][0] == 0
        assert np.array_equal(res["out_bits"], base["out_bits"])
        assert not np.isnan(codec.bf16_decode(res["out_bits"])).any()
        assert np.array_equal(res["outgoing"][(rank + 1) % P], base["outgoing"][(rank + 1) % P])


def test_partition_create_rejects_bad_sizes():
    for bad in (0, 4, 20, 256, 1024):
        with pytest.raises(pk.PkError):
            pk.pk_partition_create(bad)


def test_search_for_the_compute_unit_split():
    """The split search runs a live AG+GEMM iteration per candidate and returns the fastest; every iteration's result
    stays bit-identical to the pre-landed one."""
    from paper_2511_13940_amd import tune
    c = wl.CONFIGS["cfg2"]
    rank = 1
    inp = wl.ag_gemm_inputs(c.P, c.M, c.N, c.K, c.dtype, rank, seed=6)
    base = hz.run_ag_gemm(c.P, rank, c.M, c.N, c.K, c.dtype, inp["chunks"], inp["B_local"])
    full = np.concatenate(inp["chunks"], axis=0)
    staging = hz.elem_view(full, "bf16")
    A = staging.clone()
    B = hz.elem_view(inp["B_local"], "bf16")
    C = torch.zeros((c.M, c.N // c.P), dtype=torch.int16, device="cuda")
    flags = torch.zeros(c.P, dtype=torch.int32, device="cuda")
    counters = torch.zeros(pk.EMU_MAX_ORDER, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    epoch = [0]
    done = torch.cuda.Event()

    def launch(comp, comm, cc):
        epoch[0] += 1
        done.record(comp)
        comm.wait_event(done)
        with torch.cuda.stream(comm):
            counters.zero_()
        pk.pk_emu_deliver_chunks(c.P, c.M, c.K, 2, staging, A, flags, epoch[0], inp["order"], 0, counters, stream=comm,
                                 n_wg=4 * cc)
        pk.pk_ag_gemm(c.P, rank, c.M, c.N, c.K, c.dtype, A, B, None, None, flags, epoch[0], C, status, stream=comp,
                      comm_cus=cc)
        comp.wait_stream(comm)

    best, times = tune.search_comm_cus(launch, candidates=(8, 32, 64), iters=3, warmup=1)
    assert best in times and set(times) == {8, 32, 64} and all(t > 0 for t in times.values())
    assert status[0].item() == 0
    assert np.array_equal(hz.bits_of(C), base["C_bits"])
