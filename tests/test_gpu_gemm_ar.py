"""GPU parity of pk_gemm_ar (GEMM + all-reduce, one rank's share) against the float64 oracle, through the C ABI.

Gate as for GEMM + reduce-scatter: max |gpu - ref| / (|ref| + 1) <= 1e-2 (bf16 inputs), <= 5e-2 (fp8), plus the bound
derived from fp32 accumulation and slot additions and half a bf16 ulp.  Everything that is only moved (the blocks
handed to the other ranks, the rows received from them, flags) is compared bit for bit."""
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


def peer_rows_for(P, mp, N, seed):
    """Seeded bf16 row blocks standing in for what the other ranks hand out (any finite bit patterns will do)."""
    rng = np.random.default_rng([251113940, seed, 77])
    return wl.to_bf16_bits(rng.standard_normal((P, mp, N)).astype(np.float32) * 0.05)


def check_ar(P, rank, dtype, inp, peer_rows, res, k_local):
    ref = tp_gemm.gemm_ar(P, rank, inp["A_local"], inp["B_local"], dtype, inp["partials"], peer_rows,
                          inp.get("scale_a"), inp.get("scale_b"))
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], dtype, inp.get("scale_a"), inp.get("scale_b"))
    mp, N = ref["out"].shape
    assert res["status"][0] == 0, res["status"]
    full = res["full_bits"].reshape(P, mp, N)
    # own rows: the reduced shard
    got = codec.bf16_decode(full[rank])
    want = ref["out"]
    assert not np.isnan(got).any()
    assert gate_err(got, want) <= GATE[dtype]
    slot_mag = np.abs(ref["outgoing"][rank]) + sum(np.abs(inp["partials"][q].astype(np.float64))
                                                   for q in range(P) if q != rank)
    bound = (2 * k_local * U32 * mag[rank * mp:(rank + 1) * mp] + P * U32 * slot_mag + 2.0 ** -8 * np.abs(want)
             + 2.0 ** -133)
    assert np.all(np.abs(got - want) <= bound)
    bcast = res["bcast_bits"].reshape(P, mp, N)
    for q in range(P):
        if q == rank:
            assert np.all(bcast[q] == 0x7FC1)                       # own slot of bcast_out is unused
            continue
        assert np.array_equal(bcast[q], full[rank]), f"block handed to rank {q}"
        assert np.array_equal(full[q], peer_rows[q]), f"rows received from rank {q}"
        # scatter part as in GEMM + reduce-scatter
        assert gate_err(res["outgoing"][q], ref["outgoing"][q]) <= GATE[dtype]
    return ref


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 256, 256, 512, 0),        # one tile per shard
    (2, 2 * 348, 392, 512, 1),    # ragged rows (348 = 43 row blocks of 8 + 4) and columns
    (4, 4 * 136, 1048, 1024, 2),
    (1, 256, 256, 256, 0),        # P = 1: plain GEMM rounded to bf16, nothing handed out
    (3, 3 * 40, 16, 3 * 128, 0),
])
def test_small_tiles(dtype, P, M, N, K, rank):
    if dtype == "fp8" and (N % 16 or (K // P) % 128):
        pytest.skip("shape not valid for fp8")
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=4)
    peer = peer_rows_for(P, M // P, N, seed=rank)
    res = hz.run_gemm_ar(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], peer,
                         inp["scale_a"], inp["scale_b"], epoch=6)
    check_ar(P, rank, dtype, inp, peer, res, K // P)
    plan = res["plan"]
    assert plan.ar_flags_per_slot == -(-(M // P) // pk.AR_ROWS) * plan.tiles_n
    assert np.all(res["ar_in"] == 6)                                # own row blocks signalled, the others pre-set
    for q in range(P):
        assert np.all(res["ar_out"][q] == (0 if q == rank else 6))


@pytest.mark.parametrize("ragged", [False, True])
def test_big_tiles(ragged):
    P, rank = 2, 0
    M = 2 * (2048 - (44 if ragged else 0))
    N = 4096 - (48 if ragged else 0)
    K = 2 * 192
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=6)
    peer = peer_rows_for(P, M // P, N, seed=3)
    res = hz.run_gemm_ar(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], peer, epoch=2)
    assert res["plan"].tile_m == 256
    check_ar(P, rank, "bf16", inp, peer, res, K // P)


def test_all_ranks_end_with_the_same_full_product():
    """Every rank of one global problem on the GPU.  Pass 1 (GEMM + scatter) yields the tiles each rank sends;
    pass 2 (reduce + hand-out) yields each rank's reduced rows; in pass 3 every rank gets the others' blocks:
    all P copies of out_full are bit-identical and equal bf16(A.B) within the gate."""
    P, M, N, K = 4, 512, 384, 1024
    g = wl.global_problem(M, N, K, "bf16", seed=12)
    mp = M // P
    shares = [wl.slice_gemm_rs(g, P, r) for r in range(P)]
    zero = np.zeros((P, mp, N), np.float32)
    none = np.full((P, mp, N), 0x7FC1, np.uint16)
    sent = [hz.run_gemm_ar(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], zero, none, phases=pk.PHASE_GEMM)["outgoing"]
            for r in range(P)]

    def partials_for(r):
        out = np.zeros((P, mp, N), np.float32)
        for q in range(P):
            if q != r:
                out[q] = sent[q][r]
        return out
    blocks = []
    for r in range(P):
        res = hz.run_gemm_ar(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], partials_for(r), none,
                             phases=pk.PHASE_ALL)
        assert res["status"][0] == 0
        blocks.append(res["bcast_bits"].reshape(P, mp, N))
    fulls = []
    for r in range(P):
        handed = np.stack([none[q] if q == r else blocks[q][r] for q in range(P)])
        res = hz.run_gemm_ar(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], partials_for(r), handed)
        assert res["status"][0] == 0
        fulls.append(res["full_bits"])
    for r in range(1, P):
        assert np.array_equal(fulls[r], fulls[0])
    ref = tp_gemm.local_product(g["A"], g["B"], "bf16")
    got = codec.bf16_decode(fulls[0])
    assert gate_err(got, ref) <= GATE["bf16"]
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5)


def test_arrival_through_the_emulator_is_bit_identical_and_nan_free():
    P, rank, M, N, K = 4, 1, 4 * 384, 640, 4 * 128
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=14)
    peer = peer_rows_for(P, M // P, N, seed=8)
    base = hz.run_gemm_ar(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], peer)
    check_ar(P, rank, "bf16", inp, peer, base, K // P)
    for s in range(4):
        order = wl.arrival_order(P, rank, "random", seed=s)
        res = hz.run_gemm_ar(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], peer,
                             deliver="emu", order=order, gap_us=(0, 60)[s % 2], epoch=s + 1)
        assert res["status"][0] == 0
        assert np.array_equal(res["full_bits"], base["full_bits"]), f"order {order}"
        assert np.array_equal(res["bcast_bits"], base["bcast_bits"])
        assert not np.isnan(codec.bf16_decode(res["full_bits"])).any()
        assert np.all(res["ar_in"] == s + 1)


def test_missing_row_block_times_out_instead_of_hanging():
    P, rank, M, N, K = 2, 0, 512, 256, 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=20)
    peer = peer_rows_for(P, M // P, N, seed=1)
    res = hz.run_gemm_ar(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"], peer,
                         epoch=5, withhold_rows=(1, 7), timeout_us=2000)
    afps = res["plan"].ar_flags_per_slot
    assert res["status"][0] == pk.ERR_TIMEOUT and res["status"][1] == afps + 7 and res["status"][2] == 3
    # the own rows were still reduced and handed out
    ref = tp_gemm.gemm_ar(P, rank, inp["A_local"], inp["B_local"], "bf16", inp["partials"], peer)
    got = codec.bf16_decode(res["full_bits"].reshape(P, M // P, N)[rank])
    assert gate_err(got, ref["out"]) <= GATE["bf16"]
    assert np.all(res["ar_out"][1] == 5)
