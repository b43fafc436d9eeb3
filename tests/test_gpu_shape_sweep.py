"""Seeded sweep over random valid shapes of every op, small enough for the oracle: odd sizes around the tile edges,
P from 1 to 8, both element types, every rank position.  Gate as everywhere: max |gpu - ref| / (|ref| + 1) <= 1e-2
(bf16 inputs), <= 5e-2 (fp8 inputs)."""
import numpy as np
import pytest

from oracle import codec, tp_gemm
from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu

GATE = {"bf16": 1e-2, "fp8": 5e-2}


def gate_err(gpu, ref):
    return float(np.max(np.abs(gpu - ref) / (np.abs(ref) + 1.0)))


def cases(op, n, seed):
    """(dtype, P, rank, M, N, K) tuples valid for `op`."""
    rng = np.random.default_rng([251113940, seed, 7])
    out = []
    while len(out) < n:
        dtype = ("bf16", "fp8")[int(rng.integers(2))]
        P = int(rng.choice([1, 2, 3, 4, 5, 8]))
        rank = int(rng.integers(P))
        nv, kt = (8, 64) if dtype == "bf16" else (16, 128)
        rows = int(rng.integers(1, 420))                       # rows of one shard / of M
        cols = nv * int(rng.integers(1, 50))                   # columns of one shard / of N
        kl = kt * int(rng.integers(1, 5))                      # local k / k per chunk
        if op == "rs":          # M = P * rows, N = cols, K = P * kl
            out.append((dtype, P, rank, P * rows, cols, P * kl))
        elif op == "rs_cols":   # M = rows, N = P * cols, K = P * kl
            out.append((dtype, P, rank, rows, P * cols, P * kl))
        elif op == "ag":        # M = P * rows, N = P * cols, K = kl
            out.append((dtype, P, rank, P * rows, P * cols, kl))
        else:                   # ag_k: M = rows, N = P * cols, K = P * kl
            out.append((dtype, P, rank, rows, P * cols, P * kl))
    return out


@pytest.mark.parametrize("dtype,P,rank,M,N,K", cases("rs", 10, 1))
def test_gemm_rs(dtype, P, rank, M, N, K):
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=M + N)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], inp["scale_a"],
                         inp["scale_b"], epoch=9)
    assert res["status"][0] == 0
    ref = tp_gemm.gemm_rs(P, rank, inp["A_local"], inp["B_local"], dtype, inp["partials"], inp["scale_a"], inp["scale_b"])
    assert gate_err(codec.bf16_decode(res["out_bits"]), ref["out"]) <= GATE[dtype]
    for q in range(P):
        got = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        assert not np.isnan(got).any()
        assert gate_err(got, ref["outgoing"][q]) <= GATE[dtype]


@pytest.mark.parametrize("dtype,P,rank,M,N,K", cases("rs_cols", 8, 2))
def test_gemm_rs_cols(dtype, P, rank, M, N, K):
    inp = wl.gemm_rs_inputs(P, M * P, N, K, dtype, rank, seed=M + N)
    A = np.ascontiguousarray(inp["A_local"][:M])
    rng = np.random.default_rng(M * 7 + N)
    partials = (rng.standard_normal((P, M, N // P)) * 0.02).astype(np.float32)
    res = hz.run_gemm_rs(P, rank, M, N, K, dtype, A, inp["B_local"], partials, inp["scale_a"], inp["scale_b"], epoch=4,
                         cols=True)
    assert res["status"][0] == 0
    ref = tp_gemm.gemm_rs_cols(P, rank, A, inp["B_local"], dtype, partials, inp["scale_a"], inp["scale_b"])
    assert gate_err(codec.bf16_decode(res["out_bits"]), ref["out"]) <= GATE[dtype]
    for q in range(P):
        got = res["partials_after"][rank] if q == rank else res["outgoing"][q]
        assert not np.isnan(got).any()
        assert gate_err(got, ref["outgoing"][q]) <= GATE[dtype]


@pytest.mark.parametrize("dtype,P,rank,M,N,K", cases("ag", 10, 3))
def test_ag_gemm(dtype, P, rank, M, N, K):
    inp = wl.ag_gemm_inputs(P, M, N, K, dtype, rank, seed=M + N)
    res = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], inp["scale_a"], inp["scale_b"], epoch=2,
                         deliver="emu" if P > 1 else "pre", order=inp["order"])
    assert res["status"][0] == 0
    ref = tp_gemm.ag_gemm(P, rank, tp_gemm.gather_chunks(inp["chunks"]), inp["B_local"], dtype, inp["scale_a"],
                          inp["scale_b"])["C"]
    got = codec.bf16_decode(res["C_bits"])
    assert not np.isnan(got).any()
    assert gate_err(got, ref) <= GATE[dtype]


@pytest.mark.parametrize("dtype,P,rank,M,N,K", cases("ag_k", 8, 4))
def test_ag_gemm_k(dtype, P, rank, M, N, K):
    g = wl.global_problem(M, N, K, dtype, seed=M + N)
    kp, ns = K // P, N // P
    chunks = [np.ascontiguousarray(g["A"][:, q * kp:(q + 1) * kp]) for q in range(P)]
    B = np.ascontiguousarray(g["B"][:, rank * ns:(rank + 1) * ns])
    res = hz.run_ag_gemm_k(P, rank, M, N, K, dtype, chunks, B, g["scale_a"], g["scale_b"], epoch=6,
                           deliver="dma" if P > 1 else "pre")
    assert res["status"][0] == 0
    ref = tp_gemm.local_product(g["A"], B, dtype, g["scale_a"], g["scale_b"])
    got = codec.bf16_decode(res["C_bits"])
    assert not np.isnan(got).any()
    assert gate_err(got, ref) <= GATE[dtype]


@pytest.mark.parametrize("dtype,P,rank,M,N,K", cases("rs", 6, 5))
def test_gemm_ar(dtype, P, rank, M, N, K):
    inp = wl.gemm_rs_inputs(P, M, N, K, dtype, rank, seed=M + N)
    rng = np.random.default_rng(M + 3 * N)
    peer = wl.to_bf16_bits((rng.standard_normal((P, M // P, N)) * 0.05).astype(np.float32))
    res = hz.run_gemm_ar(P, rank, M, N, K, dtype, inp["A_local"], inp["B_local"], inp["partials"], peer, inp["scale_a"],
                         inp["scale_b"], epoch=8)
    assert res["status"][0] == 0
    ref = tp_gemm.gemm_ar(P, rank, inp["A_local"], inp["B_local"], dtype, inp["partials"], peer, inp["scale_a"], inp["scale_b"])
    full = res["full_bits"].reshape(P, M // P, N)
    assert gate_err(codec.bf16_decode(full[rank]), ref["out"]) <= GATE[dtype]
    for q in range(P):
        if q != rank:
            assert np.array_equal(full[q], peer[q])
            assert np.array_equal(res["bcast_bits"].reshape(P, M // P, N)[q], full[rank])
