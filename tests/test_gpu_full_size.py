"""Parity at the full sizes of the stated configurations, in the launch configuration bench.py times
(same entry points, same tile configuration, pre-landed peers).  The oracle evaluates a sample of whole rows:
first and last rows, both sides of every tile-row and shard boundary, and a seeded random set, so every
destination shard / source chunk and every column tile is covered.

Gate: max |gpu - ref| / (|ref| + 1) <= 1e-2 (bf16 inputs), <= 5e-2 (fp8 inputs); plus the derived bound of
the small-size tests (fp32 accumulation of k products + half a bf16 ulp)."""
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


def sample_rows(M, P, tile_m, seed, extra=24):
    mp = M // P
    rows = {0, M - 1}
    for q in range(P):
        for b in range(0, mp + 1, tile_m):
            for d in (-1, 0):
                r = q * mp + b + d
                if 0 <= r < M:
                    rows.add(r)
    rng = np.random.default_rng(seed)
    rows.update(int(x) for x in rng.integers(0, M, size=extra))
    return np.array(sorted(rows), dtype=np.int64)


@pytest.mark.parametrize("overlap", [False, True], ids=["reduce_after_gemm", "reduce_beside_gemm"])
@pytest.mark.parametrize("name,rank", [("cfg3", 0), ("cfg3", 7), ("cfg5", 3)])
def test_gemm_rs_full_size_sampled_rows(name, rank, overlap):
    """overlap: the call as bench.py's timed step makes it (PK_PHASE_OVERLAP: two GEMM launches, the reduce beside the
    second; cfg5: the narrow reduce kernel next to the fp8 GEMM)."""
    c = wl.CONFIGS[name]
    inp = wl.gemm_rs_inputs(c.P, c.M, c.N, c.K, c.dtype, rank, seed=1, order=c.order)
    res = hz.run_gemm_rs(c.P, rank, c.M, c.N, c.K, c.dtype, inp["A_local"], inp["B_local"], inp["partials"],
                         inp["scale_a"], inp["scale_b"], epoch=11, lazy=True,
                         phases=pk.PHASE_ALL | (pk.PHASE_OVERLAP if overlap else 0))
    plan = res["plan"]
    assert (plan.tile_m, plan.tile_n) == (256, 256)
    assert res["status"][0] == 0
    mp = c.M // c.P
    rows = sample_rows(c.M, c.P, plan.tile_m, seed=rank)
    own_rows, out_rows = tp_gemm.gemm_rs_rows(c.P, rank, inp["A_local"], inp["B_local"], c.dtype, inp["partials"],
                                              rows, inp["scale_a"], inp["scale_b"])
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], c.dtype, inp["scale_a"], inp["scale_b"], rows=rows)
    kl = c.K // c.P
    acc_bound = 2 * kl * U32 * mag + 1e-30
    out = codec.bf16_decode(res["out_bits"])
    for t, i in enumerate(rows):
        q = int(i // mp)
        if q == rank:
            got = out[i - rank * mp]
            want = out_rows[t]
            assert gate_err(got, want) <= GATE[c.dtype], (name, i)
            slot_mag = np.abs(own_rows[t]) + sum(np.abs(inp["partials"][p][i - rank * mp].astype(np.float64))
                                                 for p in range(c.P) if p != rank)
            assert np.all(np.abs(got - want) <= acc_bound[t] + c.P * U32 * slot_mag + 2.0 ** -8 * np.abs(want) + 2.0 ** -133)
            got32 = res["partials_t"][rank, i - rank * mp].cpu().numpy()
        else:
            got32 = res["outgoing_t"][q, i - q * mp].cpu().numpy()
        assert not np.isnan(got32).any()
        assert gate_err(got32, own_rows[t]) <= GATE[c.dtype], (name, i)
        assert np.all(np.abs(got32 - own_rows[t]) <= acc_bound[t]), (name, i)
    # every flag of every slot was signalled
    assert np.all(res["flags_in"][rank] == 11)
    for q in range(c.P):
        if q != rank:
            assert np.all(res["flags_out"][q] == 11)


@pytest.mark.parametrize("name,rank", [("cfg4", 0), ("cfg4", 5)])
def test_ag_gemm_full_size_sampled_rows(name, rank):
    c = wl.CONFIGS[name]
    inp = wl.ag_gemm_inputs(c.P, c.M, c.N, c.K, c.dtype, rank, seed=1, order=c.order)
    assert pk.pk_ag_gemm_plan(c.P, c.M, c.N, c.K, c.dtype).tile_m == 256
    # ring-order arrival through the emulator while the GEMM runs, as in a live all-gather: 32 compute units are
    # left to the communicator workgroups, the GEMM runs on the other 224
    res = hz.run_ag_gemm(c.P, rank, c.M, c.N, c.K, c.dtype, inp["chunks"], inp["B_local"], epoch=4,
                         deliver="emu", order=inp["order"], gap_us=5, fetch_A=False, comm_cus=32, n_wg=32)
    assert res["status"][0] == 0
    rows = sample_rows(c.M, c.P, 256, seed=rank)
    A = tp_gemm.gather_chunks(inp["chunks"])
    ref = tp_gemm.ag_gemm(c.P, rank, A, inp["B_local"], c.dtype, rows=rows)["C"]
    mag = tp_gemm.abs_product(A, inp["B_local"], c.dtype, rows=rows)
    got = codec.bf16_decode(res["C_bits"][rows])
    assert not np.isnan(got).any()
    assert gate_err(got, ref) <= GATE[c.dtype]
    assert np.all(np.abs(got - ref) <= 2 * c.K * U32 * mag + 2.0 ** -8 * np.abs(ref) + 2.0 ** -133)


def test_gemm_rs_at_the_papers_table3_size_sampled_rows():
    """M = N = 32768, P = 8 (section 3.1.3, Table 3): the partial slots total 4 GiB, beyond 32-bit byte offsets.
    The 7 peer slots are drawn on the device (seeded); the oracle gets the sampled rows of them."""
    P, rank, MN, kl = 8, 5, 32768, 512
    plan = pk.pk_gemm_rs_plan(P, MN, MN, P * kl, "bf16")
    assert (plan.tile_m, plan.tiles_m, plan.tiles_n) == (256, 16, 128)
    rng = np.random.default_rng([251113940, 33, 1])
    A_bits = wl.to_bf16_bits((rng.standard_normal((MN, kl)) / np.sqrt(P * kl)).astype(np.float32))
    B_bits = wl.to_bf16_bits((rng.standard_normal((kl, MN)) / np.sqrt(P * kl)).astype(np.float32))
    A, B = hz.elem_view(A_bits, "bf16"), hz.elem_view(B_bits, "bf16")
    mp = MN // P
    gen = torch.Generator(device="cuda")
    gen.manual_seed(33)
    part = torch.randn((P, mp, MN), generator=gen, device="cuda", dtype=torch.float32) * 0.02
    part[rank].fill_(float("nan"))
    outgoing = torch.full((P, mp, MN), float("nan"), dtype=torch.float32, device="cuda")
    flags_in = torch.full((P, plan.flags_per_slot), 3, dtype=torch.int32, device="cuda")
    flags_in[rank].zero_()
    flags_out = torch.zeros_like(flags_in)
    out = torch.full((mp, MN), -1, dtype=torch.int16, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    pk.pk_gemm_rs(P, rank, MN, MN, P * kl, "bf16", A, B, None, None, part, outgoing, flags_in, flags_out, 3, out,
                  pk.PHASE_ALL, status)
    torch.cuda.synchronize()
    assert status[0].item() == 0
    assert torch.all(flags_in[rank] == 3) and torch.all(flags_out[(rank + 1) % P] == 3)
    rows = sample_rows(MN, P, 256, seed=3, extra=8)[::3]
    own_rows = tp_gemm.local_product(A_bits, B_bits, "bf16", rows=rows)
    mag = tp_gemm.abs_product(A_bits, B_bits, "bf16", rows=rows)
    out_bits = hz.bits_of(out)
    for t, i in enumerate(rows):
        q, ii = int(i // mp), int(i % mp)
        got32 = (part if q == rank else outgoing)[q, ii].cpu().numpy()
        assert not np.isnan(got32).any()
        assert np.all(np.abs(got32 - own_rows[t]) <= 2 * kl * U32 * mag[t] + 1e-30), i
        if q == rank:
            slots = [part[p, ii].cpu().numpy().astype(np.float64) for p in range(P) if p != rank]
            want = own_rows[t] + sum(slots)
            got = codec.bf16_decode(out_bits[ii])
            assert gate_err(got, want) <= GATE["bf16"]
            slot_mag = np.abs(own_rows[t]) + sum(np.abs(x) for x in slots)
            assert np.all(np.abs(got - want) <= 2 * kl * U32 * mag[t] + P * U32 * slot_mag + 2.0 ** -8 * np.abs(want) + 2.0 ** -133)
    # the last row of the last slot lies beyond the 4 GiB mark of both arrays
    assert not torch.isnan(outgoing[P - 1 if rank != P - 1 else P - 2, mp - 1]).any()
