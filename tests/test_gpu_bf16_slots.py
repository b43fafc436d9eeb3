"""GPU parity of the bf16 partial-slot variant (the paper's element size for communicated tiles, s = 2) of pk_gemm_rs and
pk_gemm_ar against the float64 oracle, through the C ABI.

Gate: max |gpu - ref| / (|ref| + 1) <= 1e-2 (bf16 inputs), <= 5e-2 (fp8).  Derived bounds: a scattered bf16 tile differs
from the exact local product by the fp32 accumulation error plus half a bf16 ulp (2^-8 relative); the reduced shard by
that of the own contribution (which the oracle rounds from float64, the GPU from its fp32 accumulator: up to one whole
ulp, 2^-7 relative, when the two fall on different sides of a tie) plus the fp32 slot additions plus half an ulp of the
result."""
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
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=seed)
    inp["partials16"] = wl.to_bf16_bits(inp["partials"])
    return inp


def check(P, rank, dtype, inp, res, k_local):
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], dtype, inp["partials16"],
                          inp.get("scale_a"), inp.get("scale_b"), partial_dtype="bf16")
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], dtype, inp.get("scale_a"), inp.get("scale_b"))
    mp = ref["out"].shape[0]
    assert res["status"][0] == 0, res["status"]
    acc_bound = 2 * k_local * U32 * mag + 1e-30
    for q in range(P):
        bits = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        got, want = codec.bf16_decode(bits), ref["outgoing"][q]
        assert not np.isnan(got).any(), f"slot {q} has unwritten elements"
        assert gate_err(got, want) <= GATE[dtype]
        assert np.all(np.abs(got - want) <= acc_bound[q * mp:(q + 1) * mp] + 2.0 ** -8 * np.abs(want) + 2.0 ** -133)
    if P > 1:
        assert np.all(res["outgoing"][rank] == hz.BF16_NAN)
    got, want = codec.bf16_decode(res["out_bits"]), ref["out"]
    assert gate_err(got, want) <= GATE[dtype]
    slots = codec.bf16_decode(inp["partials16"])
    slot_mag = np.abs(ref["outgoing"][rank]) + sum(np.abs(slots[q]) for q in range(P) if q != rank)
    bound = (acc_bound[rank * mp:(rank + 1) * mp] + 2.0 ** -7 * np.abs(ref["outgoing"][rank]) + P * U32 * slot_mag
             + 2.0 ** -8 * np.abs(want) + 2.0 ** -133)
    assert np.all(np.abs(got - want) <= bound)
    return ref


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 256, 256, 512, 1),
    (2, 704, 392, 512, 0),        # ragged rows and columns, 128-tiles
    (4, 4 * 136, 1048, 1024, 3),
    (1, 256, 256, 256, 0),
    (3, 3 * 40, 16, 3 * 128, 2),  # runtime-P reduce
])
def test_small_tiles(dtype, P, M, N, K, rank):
    if dtype == "fp8" and (N % 16 or (K // P) % 128):
        pytest.skip("shape not valid for fp8")
    inp = inputs(P, M, N, K, dtype, rank, seed=7)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials16"],
                         inp["scale_a"], inp["scale_b"], epoch=4, partial_dtype="bf16")
    check(P, rank, dtype, inp, res, K // P)
    assert np.all(res["flags_in"][rank] == 4)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("ragged", [False, True])
def test_big_tiles(dtype, ragged):
    P, rank = 2, 1
    M = 2 * (2048 - (40 if ragged else 0))
    N = 4096 - (48 if ragged else 0)
    K = 2 * (256 if dtype == "fp8" else 192)
    inp = inputs(P, M, N, K, dtype, rank, seed=8)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials16"],
                         inp["scale_a"], inp["scale_b"], epoch=3, partial_dtype="bf16")
    assert res["plan"].tile_m == 256
    check(P, rank, dtype, inp, res, K // P)


def test_all_ranks_with_real_bf16_tiles():
    P, M, N, K = 4, 512, 384, 1024
    g = wl.global_problem(M, N, K, "bf16", seed=15)
    mp = M // P
    shares = [wl.slice_gemm_rs(g, P, r) for r in range(P)]
    zero = np.zeros((P, mp, N), np.uint16)
    sent = [hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], zero, phases=pk.PHASE_GEMM,
                           partial_dtype="bf16")["outgoing"] for r in range(P)]
    shards = []
    for r in range(P):
        partials = np.stack([zero[q] if q == r else sent[q][r] for q in range(P)])
        res = hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], partials, partial_dtype="bf16")
        assert res["status"][0] == 0
        shards.append(codec.bf16_decode(res["out_bits"]))
    full = tp_gemm.local_product(g["A"], g["B"], "bf16")
    stacked = np.concatenate(shards, axis=0)
    assert gate_err(stacked, full) <= GATE["bf16"]
    # P contributions rounded to bf16 (each at most half an ulp of a partial sum) plus the final rounding
    part_mag = sum(np.abs(tp_gemm.local_product(a, b, "bf16")) for a, b in shares)
    assert np.all(np.abs(stacked - full) <= 2.0 ** -8 * part_mag + 2.0 ** -8 * np.abs(full) + 1e-5)


def test_arrival_through_the_emulator_is_bit_identical():
    P, rank, M, N, K = 4, 2, 4 * 384, 640, 4 * 128
    inp = inputs(P, M, N, K, "bf16", rank, seed=16)
    base = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials16"], partial_dtype="bf16")
    check(P, rank, "bf16", inp, base, K // P)
    for s in range(3):
        order = wl.arrival_order(P, rank, "random", seed=s)
        res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials16"], deliver="emu",
                             order=order, gap_us=(0, 80, 0)[s], epoch=s + 1, partial_dtype="bf16")
        assert res["status"][0] == 0
        assert np.array_equal(res["out_bits"], base["out_bits"])
        assert not np.isnan(codec.bf16_decode(res["out_bits"])).any()


def test_gemm_ar_with_bf16_slots():
    P, rank, M, N, K = 4, 1, 4 * 136, 1048, 1024
    inp = inputs(P, M, N, K, "bf16", rank, seed=17)
    rng = np.random.default_rng(5)
    peer = wl.to_bf16_bits(rng.standard_normal((P, M // P, N)).astype(np.float32) * 0.05)
    res = hz.run_gemm_ar(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials16"], peer,
                         partial_dtype="bf16")
    assert res["status"][0] == 0
    ref = tp_gemm.gemm_ar(P, rank, inp["A_local"], inp["B_local"], "bf16", inp["partials16"], peer, partial_dtype="bf16")
    full = res["full_bits"].reshape(P, M // P, N)
    assert gate_err(codec.bf16_decode(full[rank]), ref["out"]) <= GATE["bf16"]
    for q in range(P):
        if q != rank:
            assert np.array_equal(full[q], peer[q])
            assert np.array_equal(res["bcast_bits"].reshape(P, M // P, N)[q], full[rank])
