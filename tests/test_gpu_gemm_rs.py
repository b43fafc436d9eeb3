"""GPU parity of pk_gemm_rs against the float64 oracle, through the C ABI.

Gate (the stated contract): max |gpu - ref| / (|ref| + 1) <= 1e-2 for bf16 inputs, <= 5e-2 for fp8.
On top of it a bound derived from the arithmetic: the fp32 tiles differ from the exact sum by at most
2*k*2^-24 * sum|a||b| (fp32 accumulation of k products, any order), and the bf16 result by that plus the
fp32 slot additions plus half a bf16 ulp (2^-8 relative)."""
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


def check_rs(P, rank, dtype, inp, res, k_local):
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], dtype, inp["partials"],
                          inp.get("scale_a"), inp.get("scale_b"))
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], dtype, inp.get("scale_a"), inp.get("scale_b"))
    M, N = ref["own"].shape
    mp = M // P
    assert res["status"][0] == 0, res["status"]
    acc_bound = 2 * k_local * U32 * mag + 1e-30
    # scattered fp32 tiles: every destination slot equals its row block of the local product
    for q in range(P):
        got = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        want = ref["outgoing"][q]
        assert not np.isnan(got).any(), f"slot {q} has unwritten elements"
        assert gate_err(got, want) <= GATE[dtype]
        assert np.all(np.abs(got - want) <= acc_bound[q * mp:(q + 1) * mp]), f"slot {q}"
    # own slot of outgoing is documented as unused: still poison
    if P > 1:
        assert np.isnan(res["outgoing"][rank]).all()
    # reduced shard
    got = codec.bf16_decode(res["out_bits"])
    want = ref["out"]
    assert gate_err(got, want) <= GATE[dtype]
    slot_mag = np.abs(ref["outgoing"][rank]) + sum(np.abs(inp["partials"][q].astype(np.float64))
                                                   for q in range(P) if q != rank)
    bound = acc_bound[rank * mp:(rank + 1) * mp] + P * U32 * slot_mag + 2.0 ** -8 * np.abs(want) + 2.0 ** -133
    assert np.all(np.abs(got - want) <= bound)
    # flags: every tile of every slot was signalled with the epoch
    return ref


@pytest.mark.parametrize("rank", [0, 1])
def test_cfg1_every_rank(rank):
    c = wl.CONFIGS["cfg1"]
    inp = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, rank, seed=0)
    res = hz.run_gemm_rs(c.P, rank, c.M, c.N, c.K, c.dtype, inp["A_local"], inp["B_local"], inp["partials"], epoch=7)
    check_rs(c.P, rank, c.dtype, inp, res, c.K // c.P)
    assert np.all(res["flags_out"][1 - rank] == 7) and np.all(res["flags_in"][rank] == 7)
    assert np.all(res["flags_out"][rank] == 0)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("P,M,N,K,rank", [
    (2, 704, 392, 512, 1),        # 128-tiles: 3 tile rows per shard with a ragged last one, ragged columns
    (4, 4 * 136, 1048, 1024, 2),  # shard smaller than two tiles; 9 column tiles, last one 24 wide
    (1, 256, 256, 256, 0),        # P = 1: plain GEMM rounded to bf16
    (3, 3 * 40, 16, 3 * 128, 0),  # a single partial tile per shard, odd P (runtime-P reduce)
])
def test_ragged_small_tiles(dtype, P, M, N, K, rank):
    if dtype == "fp8" and (N % 16 or (K // P) % 128):
        pytest.skip("shape not valid for fp8")
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=3)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"],
                         inp["scale_a"], inp["scale_b"], epoch=2)
    assert res["plan"].tile_m == 128
    check_rs(P, rank, dtype, inp, res, K // P)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("ragged", [False, True])
def test_big_tiles(dtype, ragged):
    """Enough tiles for the 256 x 256 configuration (2 x 8 x 16 = 256 tiles), optionally with ragged edges."""
    P, rank = 2, 1
    M = 2 * (2048 - (40 if ragged else 0))
    N = 4096 - (48 if ragged else 0)
    K = 2 * (256 if dtype == "fp8" else 192)
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=5)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"],
                         inp["scale_a"], inp["scale_b"], epoch=3)
    assert res["plan"].tile_m == 256 and res["plan"].tile_n == 256
    check_rs(P, rank, dtype, inp, res, K // P)


def test_all_ranks_linearity_and_shard_concatenation():
    """Run every rank of one global problem on the GPU, feeding each rank the tiles the others sent
    (their `outgoing` slots): the stacked shards equal bf16(A.B) of the unsharded problem."""
    P, M, N, K = 4, 512, 384, 1024
    g = wl.global_problem(M, N, K, "bf16", seed=11)
    mp = M // P
    shares = [wl.slice_gemm_rs(g, P, r) for r in range(P)]
    zero = np.zeros((P, mp, N), np.float32)
    sent = []
    for r in range(P):   # pass 1: only the GEMM + scatter phase
        res = hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], zero, phases=pk.PHASE_GEMM)
        sent.append((res["outgoing"], res["partials_after"][r]))
    # linearity on the GPU's own fp32 tiles: sum over ranks of the local products = unsharded product
    full = tp_gemm.local_product(g["A"], g["B"], "bf16")
    total = np.zeros((M, N))
    for r in range(P):
        own = np.concatenate([sent[r][1] if q == r else sent[r][0][q] for q in range(P)], axis=0)
        total += own.astype(np.float64)
    assert np.max(np.abs(total - full)) <= 2 * K * U32 * np.max(tp_gemm.abs_product(g["A"], g["B"], "bf16"))
    shards = []
    for r in range(P):   # pass 2: the full op with the peers' real tiles
        partials = np.zeros((P, mp, N), np.float32)
        for q in range(P):
            if q != r:
                partials[q] = sent[q][0][r]
        res = hz.run_gemm_rs(P, r, M, N, K, "bf16", shares[r][0], shares[r][1], partials)
        shards.append(codec.bf16_decode(res["out_bits"]))
    stacked = np.concatenate(shards, axis=0)
    assert gate_err(stacked, full) <= GATE["bf16"]
    assert np.all(np.abs(stacked - full) <= 2.0 ** -8 * np.abs(full) + 1e-5)


def test_arrival_order_independence_and_no_early_reads():
    """Peers' tiles land through the emulator in several orders and with gaps, into NaN-poisoned slots:
    the result must be bit-identical to the pre-landed run and contain no NaN."""
    P, rank, M, N, K = 4, 1, 4 * 384, 640, 4 * 128
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=13)
    base = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"])
    check_rs(P, rank, "bf16", inp, base, K // P)
    for s in range(10):
        order = wl.arrival_order(P, rank, "random", seed=s)
        res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"],
                             deliver="emu", order=order, gap_us=(0, 50, 300)[s % 3], epoch=s + 1)
        assert res["status"][0] == 0
        assert np.array_equal(res["out_bits"], base["out_bits"]), f"order {order}"
        assert not np.isnan(codec.bf16_decode(res["out_bits"])).any()


def test_epoch_reuse_without_reset():
    """Back-to-back calls on the SAME flag arrays with increasing epochs (no reset in between), across
    the signed and unsigned wrap-around points of the 32-bit counter."""
    P, rank, M, N, K = 2, 0, 512, 256, 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=17)
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], "bf16", inp["partials"])
    plan = pk.pk_gemm_rs_plan(P, M, N, K, "bf16")
    mp = M // P
    A, B = hz.elem_view(inp["A_local"], "bf16"), hz.elem_view(inp["B_local"], "bf16")
    part = hz.dev(inp["partials"])
    outgoing = torch.zeros((P, mp, N), dtype=torch.float32, device="cuda")
    flags_in = torch.zeros((P, plan.flags_per_slot), dtype=torch.int32, device="cuda")
    flags_out = torch.zeros_like(flags_in)
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    out = torch.zeros((mp, N), dtype=torch.int16, device="cuda")
    for e in [1, 2, 3, 0x7FFFFFFF, 0x80000000, 0x80000001, 0xFFFFFFFF, 0, 1]:
        signed = e if e < 2 ** 31 else e - 2 ** 32
        out.fill_(-1)
        part[rank].fill_(float("nan"))
        flags_in[1].fill_(signed)
        torch.cuda.synchronize()
        pk.pk_gemm_rs(P, rank, M, N, K, "bf16", A, B, None, None, part, outgoing, flags_in, flags_out, e, out,
                      pk.PHASE_ALL, status, 0)
        torch.cuda.synchronize()
        assert status[0].item() == 0
        assert np.array_equal(hz.bits_of(out), ref["out_bf16"]) or \
            gate_err(codec.bf16_decode(hz.bits_of(out)), ref["out"]) <= GATE["bf16"]
        assert torch.all(flags_out[1] == signed) and torch.all(flags_in[0] == signed)


def test_missing_flag_times_out_instead_of_hanging():
    P, rank, M, N, K = 2, 0, 512, 256, 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=19)
    res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", inp["A_local"], inp["B_local"], inp["partials"],
                         epoch=9, withhold=(1, 3), timeout_us=2000)
    assert res["status"][0] == pk.ERR_TIMEOUT and res["status"][1] == 3 and res["status"][2] == 2
    # every other tile was still reduced
    plan = res["plan"]
    got = codec.bf16_decode(res["out_bits"]).reshape(plan.tiles_m, plan.tile_m, plan.tiles_n, plan.tile_n)
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], "bf16", inp["partials"])["out"]
    ref = ref.reshape(plan.tiles_m, plan.tile_m, plan.tiles_n, plan.tile_n)
    for t in range(plan.tiles_m * plan.tiles_n):
        if t != 3:
            tm, tn = divmod(t, plan.tiles_n)
            assert gate_err(got[tm, :, tn], ref[tm, :, tn]) <= GATE["bf16"]


def test_reduce_phase_alone_matches_closed_forms():
    """PK_PHASE_REDUCE on hand-made slots: constants sum to their total, +x/-x pairs cancel."""
    P, rank, M, N, K = 4, 2, 4 * 160, 264, 4 * 64
    mp = M // P
    consts = np.array([1.5, -2.25, 4.0, 0.125], np.float32)
    partials = np.broadcast_to(consts[:, None, None], (P, mp, N)).copy()
    plan = pk.pk_gemm_rs_plan(P, M, N, K, "bf16")
    part = hz.dev(partials)
    out = torch.zeros((mp, N), dtype=torch.int16, device="cuda")
    flags = torch.full((P, plan.flags_per_slot), 4, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    pk.pk_gemm_rs(P, rank, M, N, K, "bf16", None, None, None, None, part, None, flags, None, 4, out,
                  pk.PHASE_REDUCE, status)
    torch.cuda.synchronize()
    assert status[0].item() == 0
    assert np.all(codec.bf16_decode(hz.bits_of(out)) == 3.375)
    x = np.random.default_rng(1).standard_normal((mp, N)).astype(np.float32)
    part.copy_(torch.from_numpy(np.stack([x, -x, 2 * x, -2 * x])))
    pk.pk_gemm_rs(P, rank, M, N, K, "bf16", None, None, None, None, part, None, flags, None, 4, out,
                  pk.PHASE_REDUCE, status)
    torch.cuda.synchronize()
    assert np.all(codec.bf16_decode(hz.bits_of(out)) == 0.0)
