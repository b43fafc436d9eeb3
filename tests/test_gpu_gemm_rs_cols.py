"""GPU parity of pk_gemm_rs_cols (GEMM + reduce-scatter along the last dimension) against the float64 oracle, through
the C ABI.  Gates and derived bounds as for pk_gemm_rs."""
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
    """Operands as for GEMM + reduce-scatter; peer slots [P][M][N/P] of the magnitude of a true partial."""
    inp = wl.gemm_rs_inputs(P, M * P, N, K, dtype, rank, seed=seed)             # A_local comes out (M*P) x K/P: take M rows
    inp["A_local"] = np.ascontiguousarray(inp["A_local"][:M])
    rng = np.random.default_rng([251113940, seed, 99])
    inp["partials"] = (rng.standard_normal((P, M, N // P)) * np.sqrt(K / P) / K).astype(np.float32)
    return inp


def check(P, rank, dtype, inp, res, k_local, partial_dtype="f32"):
    slots = inp["partials16"] if partial_dtype == "bf16" else inp["partials"]
    ref = tp_gemm.gemm_rs_cols(P, rank, inp["A_local"], inp["B_local"], dtype, slots, inp.get("scale_a"), inp.get("scale_b"),
                               partial_dtype=partial_dtype)
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], dtype, inp.get("scale_a"), inp.get("scale_b"))
    M, N = ref["own"].shape
    ns = N // P
    assert res["status"][0] == 0, res["status"]
    acc_bound = 2 * k_local * U32 * mag + 1e-30
    half_ulp = 2.0 ** -8 if partial_dtype == "bf16" else 0.0
    for q in range(P):
        got = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        if partial_dtype == "bf16":
            got = codec.bf16_decode(got)
        want = ref["outgoing"][q]
        assert not np.isnan(got).any(), f"slot {q} has unwritten elements"
        assert gate_err(got, want) <= GATE[dtype]
        assert np.all(np.abs(got - want) <= acc_bound[:, q * ns:(q + 1) * ns] + half_ulp * np.abs(want) + 2.0 ** -133), f"slot {q}"
    got, want = codec.bf16_decode(res["out_bits"]), ref["out"]
    assert got.shape == (M, ns)
    assert gate_err(got, want) <= GATE[dtype]
    vals = codec.bf16_decode(slots) if partial_dtype == "bf16" else slots.astype(np.float64)
    slot_mag = np.abs(ref["outgoing"][rank]) + sum(np.abs(vals[q]) for q in range(P) if q != rank)
    bound = (acc_bound[:, rank * ns:(rank + 1) * ns] + 2 * half_ulp * np.abs(ref["outgoing"][rank]) + P * U32 * slot_mag
             + 2.0 ** -8 * np.abs(want) + 2.0 ** -133)
    assert np.all(np.abs(got - want) <= bound)
    plan = res["plan"]
    assert np.all(res["flags_in"][rank] == res["epoch"])
    for q in range(P):
        if q != rank:
            assert np.all(res["flags_out"][q] == res["epoch"])
    assert plan.flags_per_slot == plan.tiles_m * plan.tiles_n
    return ref


def run(P, rank, M, N, K, dtype, inp, epoch=3, **kw):
    slots = inp["partials16"] if kw.get("partial_dtype") == "bf16" else inp["partials"]
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], slots, inp["scale_a"], inp["scale_b"],
                         epoch=epoch, cols=True, **kw)
    res["epoch"] = epoch
    return res


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 256, 2 * 256, 512, 0),       # 128-tiles, two column tiles per block
    (2, 300, 2 * 200, 512, 1),       # ragged rows; column block 200 = one full tile + 72 columns
    (4, 136, 4 * 264, 1024, 2),      # M not a multiple of P; 3 column tiles per block, last one 8 wide
    (1, 256, 256, 256, 0),           # P = 1
    (3, 40, 3 * 16, 3 * 128, 1),     # odd P, a single partial tile per block
])
def test_small_tiles(dtype, P, M, N, K, rank):
    if dtype == "fp8" and ((N // P) % 16 or (K // P) % 128):
        pytest.skip("shape not valid for fp8")
    inp = inputs(P, M, N, K, dtype, rank, seed=9)
    res = run(P, rank, M, N, K, dtype, inp)
    assert res["plan"].tile_m == 128
    check(P, rank, dtype, inp, res, K // P)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("ragged", [False, True])
def test_big_tiles(dtype, ragged):
    P, rank = 2, 1
    M = 4096 - (40 if ragged else 0)
    N = 2 * (2048 - (48 if ragged else 0))
    K = 2 * (256 if dtype == "fp8" else 192)
    inp = inputs(P, M, N, K, dtype, rank, seed=10)
    res = run(P, rank, M, N, K, dtype, inp)
    assert res["plan"].tile_m == 256 and res["plan"].tile_n == 256
    check(P, rank, dtype, inp, res, K // P)


def test_bf16_slots_and_emulated_arrival():
    P, rank, M, N, K = 4, 3, 384, 4 * 320, 4 * 128
    inp = inputs(P, M, N, K, "bf16", rank, seed=11)
    inp["partials16"] = wl.to_bf16_bits(inp["partials"])
    base = run(P, rank, M, N, K, "bf16", inp, partial_dtype="bf16")
    check(P, rank, "bf16", inp, base, K // P, partial_dtype="bf16")
    base32 = run(P, rank, M, N, K, "bf16", inp)
    check(P, rank, "bf16", inp, base32, K // P)
    for s in range(3):
        order = wl.arrival_order(P, rank, "random", seed=s)
        res = run(P, rank, M, N, K, "bf16", inp, epoch=s + 1, deliver="emu", order=order, gap_us=(0, 60, 0)[s])
        assert res["status"][0] == 0
        assert np.array_equal(res["out_bits"], base32["out_bits"])
        assert not np.isnan(codec.bf16_decode(res["out_bits"])).any()


def test_all_ranks_column_blocks_concatenate_to_the_full_product():
    P, M, N, K = 4, 320, 4 * 192, 1024
    g = wl.global_problem(M, N, K, "bf16", seed=17)
    ns = N // P
    shares = [wl.slice_gemm_rs(g, P, r) for r in range(P)]
    zero = np.zeros((P, M, ns), np.float32)
    sent = [hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], zero, phases=pk.PHASE_GEMM, cols=True)["outgoing"]
            for r in range(P)]
    blocks = []
    for r in range(P):
        partials = np.stack([zero[q] if q == r else sent[q][r] for q in range(P)])
        res = hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], partials, cols=True)
        assert res["status"][0] == 0
        blocks.append(codec.bf16_decode(res["out_bits"]))
    full = tp_gemm.local_product(g["A"], g["B"], "bf16")
    stacked = np.concatenate(blocks, axis=1)
    assert gate_err(stacked, full) <= GATE["bf16"]
    assert np.all(np.abs(stacked - full) <= 2.0 ** -8 * np.abs(full) + 1e-5)
