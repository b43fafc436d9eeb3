"""pk_gemm_rs with PK_PHASE_OVERLAP (the reduce beside the second part of the GEMM, on the library's own stream):
parity against the float64 oracle and bit-identity with the plain call, on shapes whose schedule has more rounds than
the own block takes (so that the two-launch path is really taken) and on one where the flag must fall back."""
import numpy as np
import pytest
import torch

from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz
from tests.test_gpu_bf16_slots import check as check16
from tests.test_gpu_gemm_rs import check_rs

pytestmark = pytest.mark.gpu

OVERLAP = pk.PHASE_ALL | pk.PHASE_OVERLAP

CASES = [
    # P, rank, M, N, K, dtype, tile
    (8, 3, 4096, 2048, 2048, "bf16", 128),            # 512 tiles of 128: 2 rounds, own block = a quarter of the first
    (8, 7, 8192, 4096, 4096, "bf16", 256),            # 512 tiles of 256, last rank: the row rotation wraps around
    (4, 1, 4400, 2056, 1024, "bf16", 128),            # 9 ragged tile rows per block (not a multiple of the band), ragged columns
    (8, 2, 8192, 4096, 8192, "fp8", 256),             # 256x256 fp8 kernel: the narrow reduce kernel runs beside it
    (4, 3, 8192, 4096 + 272, 4096, "fp8", 256),       # the same with a ragged last column tile
    (2, 0, 4096, 8192, 1024, "bf16", 256),            # own block = half of all tiles, two rounds of four
]


@pytest.mark.parametrize("P,rank,M,N,K,dtype,tile", CASES)
@pytest.mark.parametrize("deliver", ["pre", "emu"])
def test_overlapped_reduce_matches_oracle_and_plain_call(P, rank, M, N, K, dtype, tile, deliver):
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=11)
    kw = dict(scale_a=inp.get("scale_a"), scale_b=inp.get("scale_b"), deliver=deliver, order=inp["order"], epoch=5,
              timeout_us=2_000_000)
    plain = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], **kw)
    over = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], phases=OVERLAP, **kw)
    assert over["plan"].tile_m == tile
    check_rs(P, rank, dtype, inp, over, K // P)
    assert np.array_equal(over["out_bits"], plain["out_bits"])
    for q in range(P):
        if q != rank:
            assert np.array_equal(over["outgoing"][q].view(np.uint32), plain["outgoing"][q].view(np.uint32)), q
    assert np.array_equal(over["partials_after"][rank].view(np.uint32), plain["partials_after"][rank].view(np.uint32))
    assert np.array_equal(over["flags_out"], plain["flags_out"]) and np.array_equal(over["flags_in"], plain["flags_in"])


def test_flag_falls_back_when_the_own_block_takes_every_round():
    """One round in all (cfg1-sized problem): the call runs as the plain one does."""
    c = wl.CONFIGS["cfg1"]
    inp = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, 1, seed=2)
    res = hz.run_gemm_rs(c.P, 1, c.M, c.N, c.K, c.dtype, inp["A_local"], inp["B_local"], inp["partials"], phases=OVERLAP)
    check_rs(c.P, 1, c.dtype, inp, res, c.K // c.P)


def test_bf16_slots_and_repeated_calls_with_rising_epochs():
    """bf16 partial slots next to the bf16 kernel, three calls in a row on the same buffers (the second stream and its
    events are reused; every call's reduce must see that call's own block)."""
    P, rank, M, N, K = 8, 4, 4096, 2048, 2048
    outs = []
    for seed, epoch in ((1, 1), (2, 2), (1, 3)):
        inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=seed)
        p16 = wl.to_bf16_bits(inp["partials"])
        res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], p16, epoch=epoch, phases=OVERLAP,
                             partial_dtype="bf16")
        ref = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], p16, epoch=epoch, partial_dtype="bf16")
        assert res["status"][0] == 0 and ref["status"][0] == 0
        check16(P, rank, "bf16", dict(inp, partials16=p16), res, K // P)
        assert np.array_equal(res["out_bits"], ref["out_bits"])
        outs.append(res["out_bits"])
    assert np.array_equal(outs[0], outs[2]) and not np.array_equal(outs[0], outs[1])


def test_overlap_flag_needs_both_phases():
    t = torch.zeros(4096, dtype=torch.int32, device="cuda")
    for phases in (pk.PHASE_GEMM | pk.PHASE_OVERLAP, pk.PHASE_REDUCE | pk.PHASE_OVERLAP, pk.PHASE_OVERLAP):
        with pytest.raises(pk.PkError) as e:
            pk.pk_gemm_rs(2, 0, 256, 256, 512, "bf16", t, t, None, None, t, t, t, t, 1, t, phases, t)
        assert e.value.code == pk.ERR_ARG


def test_overlap_on_a_compute_unit_partition_with_live_peers():
    """The GEMM launches on the compute stream of a partition (224 workgroups), the peers' partials arrive through the
    communicator stream while it runs, the reduce on the library's own stream: same bits as the plain pre-landed call."""
    P, rank, M, N, K = 4, 3, 4096, 4096, 4 * 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=21)
    base = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"])
    check_rs(P, rank, "bf16", inp, base, K // P)
    comp, comm = pk.pk_partition_create(32)
    try:
        for i, n_wg in enumerate([32, 128]):
            order = wl.arrival_order(P, rank, "random", seed=i)
            res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], deliver="emu",
                                 order=order, epoch=i + 1, comm_cus=32, n_wg=n_wg, partition=(comp, comm), phases=OVERLAP,
                                 timeout_us=2_000_000)
            assert res["status"][0] == 0
            assert np.array_equal(res["out_bits"], base["out_bits"])
            for q in range(P):
                if q != rank:
                    assert np.array_equal(res["outgoing"][q].view(np.uint32), base["outgoing"][q].view(np.uint32))
    finally:
        torch.cuda.synchronize()
        pk.pk_partition_destroy(comp, comm)


def test_overlap_flag_with_a_single_rank_is_the_plain_gemm():
    inp = wl.gemm_rs_inputs(1, 1024, 2048, 512, "bf16", 0, seed=4)
    res = hz.run_gemm_rs(1, 0, 1024, 2048, 512, "bf16", inp["A_local"], inp["B_local"], inp["partials"], phases=OVERLAP)
    check_rs(1, 0, "bf16", inp, res, 512)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_overlap_flag_with_a_k_contiguous_second_operand(dtype):
    """bf16: the narrow reduce kernel beside the k-contiguous GEMM kernel; fp8: no room beside that kernel, plain order."""
    P, rank, M, N, K = 8, 6, 8192, 4096, 8192
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=13)
    Bt = np.ascontiguousarray(inp["B_local"].T)
    kw = dict(scale_a=inp.get("scale_a"), scale_b=inp.get("scale_b"), epoch=3)
    plain = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], **kw)
    over = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], Bt, inp["partials"], phases=OVERLAP, b_layout="nk", **kw)
    assert over["plan"].tile_m == 256
    check_rs(P, rank, dtype, inp, over, K // P)
    assert np.array_equal(over["out_bits"], plain["out_bits"])
