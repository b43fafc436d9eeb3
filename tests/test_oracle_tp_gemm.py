"""Pins for the oracle's GEMM+RS / AG+GEMM definitions: exact integer and rational
brute force, textbook special cases, the linearity and shard-concatenation
identities.  None of the expected values below is produced by the oracle."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import codec, tp_gemm
from paper_2511_13940_amd import workloads as wl


def _int_bits(x, dtype):
    """Small integers are exact in both storage formats."""
    if dtype == "bf16":
        return wl.to_bf16_bits(x.astype(np.float32))
    import torch
    return torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def _brute_int(a, b):
    """Triple loop in Python integers."""
    m, k = a.shape
    n = b.shape[1]
    return [[sum(int(a[i, t]) * int(b[t, j]) for t in range(k)) for j in range(n)] for i in range(m)]


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (2, 3, 5), (7, 5, 3), (17, 13, 11), (4, 9, 16)])
def test_local_product_integer_brute_force(dtype, m, n, k):
    a = wl.small_int_matrix((m, k), 11, m * 100 + k)
    b = wl.small_int_matrix((k, n), 12, n * 100 + k)
    got = tp_gemm.local_product(_int_bits(a, dtype), _int_bits(b, dtype), dtype)
    assert got.shape == (m, n)
    assert np.array_equal(got, np.array(_brute_int(a, b), dtype=np.float64))


def test_local_product_rational_brute_force_bf16():
    """Random bf16 inputs, exact rational dot products; float64 accumulation of 11 terms
    is within a few ulp of the exact value."""
    m, n, k = 5, 7, 11
    rng = np.random.default_rng(5)
    a_bits = wl.to_bf16_bits(rng.standard_normal((m, k)).astype(np.float32))
    b_bits = wl.to_bf16_bits(rng.standard_normal((k, n)).astype(np.float32))
    af = [[Fraction(float(v)) for v in row] for row in codec.bf16_decode(a_bits)]
    bf = [[Fraction(float(v)) for v in row] for row in codec.bf16_decode(b_bits)]
    got = tp_gemm.local_product(a_bits, b_bits, "bf16")
    for i in range(m):
        for j in range(n):
            exact = sum(af[i][t] * bf[t][j] for t in range(k))
            mag = sum(abs(af[i][t] * bf[t][j]) for t in range(k))
            assert abs(Fraction(float(got[i, j])) - exact) <= mag * Fraction(k, 2 ** 52)


def test_local_product_special_cases():
    rng = np.random.default_rng(9)
    a = rng.integers(-3, 4, size=(6, 6)).astype(np.float32)
    eye = np.eye(6, dtype=np.float32)
    perm = eye[:, [2, 0, 5, 1, 4, 3]]
    ab = wl.to_bf16_bits(a)
    assert np.array_equal(tp_gemm.local_product(ab, wl.to_bf16_bits(eye), "bf16"), a)
    assert np.array_equal(tp_gemm.local_product(wl.to_bf16_bits(eye), ab, "bf16"), a)
    # A.Perm permutes columns, Perm.A permutes rows: catches a transposed operand
    assert np.array_equal(tp_gemm.local_product(ab, wl.to_bf16_bits(perm), "bf16"), a[:, [2, 0, 5, 1, 4, 3]])
    assert np.array_equal(tp_gemm.local_product(wl.to_bf16_bits(perm.T), ab, "bf16"), a[[2, 0, 5, 1, 4, 3], :])
    ones = np.ones((6, 4), dtype=np.float32)
    assert np.array_equal(tp_gemm.local_product(ab, wl.to_bf16_bits(ones), "bf16"),
                          np.repeat(a.sum(axis=1, keepdims=True), 4, axis=1))


def test_scales_are_applied_once_fp8():
    a = wl.small_int_matrix((3, 8), 1, 1)
    b = wl.small_int_matrix((8, 5), 1, 2)
    sa, sb = np.float32(0.25), np.float32(8.0)
    got = tp_gemm.local_product(_int_bits(a, "fp8"), _int_bits(b, "fp8"), "fp8", sa, sb)
    assert np.array_equal(got, 2.0 * np.array(_brute_int(a, b), dtype=np.float64))
    sa, sb = np.float32(0.1), np.float32(0.3)   # not exactly representable: taken as float32 values
    got = tp_gemm.local_product(_int_bits(a, "fp8"), _int_bits(b, "fp8"), "fp8", sa, sb)
    s = Fraction(float(sa)) * Fraction(float(sb))
    ref = np.array([[float(s * v) for v in row] for row in _brute_int(a, b)])
    assert np.allclose(got, ref, rtol=1e-15, atol=0)


@pytest.mark.parametrize("P,M,N,K", [(2, 4, 3, 6), (3, 6, 5, 9), (4, 8, 2, 8)])
def test_gemm_rs_integer_brute_force_all_ranks(P, M, N, K):
    """Every rank run on one global integer problem with true partials: each reduced
    shard equals the rows of the unsharded product, and the outgoing slots are the
    right row blocks of the local product."""
    A = wl.small_int_matrix((M, K), 21, 1)
    B = wl.small_int_matrix((K, N), 21, 2)
    full = np.array(_brute_int(A, B), dtype=np.float64)
    kp, mp = K // P, M // P
    local = [np.array(_brute_int(A[:, r * kp:(r + 1) * kp], B[r * kp:(r + 1) * kp, :]), dtype=np.float64)
             for r in range(P)]
    assert np.array_equal(sum(local), full)                       # linearity, in integers
    for r in range(P):
        partials = np.zeros((P, mp, N), dtype=np.float32)
        for q in range(P):
            if q != r:
                partials[q] = local[q][r * mp:(r + 1) * mp]
        partials[r] = 12345.0                                      # must be ignored
        res = tp_gemm.gemm_rs(P, r, _int_bits(A[:, r * kp:(r + 1) * kp], "bf16"),
                              _int_bits(B[r * kp:(r + 1) * kp, :], "bf16"), "bf16", partials)
        assert np.array_equal(res["own"], local[r])
        for q in range(P):
            assert np.array_equal(res["outgoing"][q], local[r][q * mp:(q + 1) * mp])
        assert np.array_equal(res["out"], full[r * mp:(r + 1) * mp])
        assert np.array_equal(codec.bf16_decode(res["out_bf16"]), full[r * mp:(r + 1) * mp])


@pytest.mark.parametrize("P,M,N,K", [(2, 4, 3, 6), (4, 8, 2, 8)])
def test_gemm_ar_integer_brute_force_all_ranks(P, M, N, K):
    """GEMM + all-reduce on one global integer problem: rank r's reduced rows are rows R_r of the
    unsharded product; handing every rank's rounded block to every other rank leaves each rank with
    the same full product (here exactly representable in bf16)."""
    A = wl.small_int_matrix((M, K), 33, 1)
    B = wl.small_int_matrix((K, N), 33, 2)
    full = np.array(_brute_int(A, B), dtype=np.float64)
    kp, mp = K // P, M // P
    local = [np.array(_brute_int(A[:, r * kp:(r + 1) * kp], B[r * kp:(r + 1) * kp, :]), dtype=np.float64)
             for r in range(P)]
    shares = [(_int_bits(A[:, r * kp:(r + 1) * kp], "bf16"), _int_bits(B[r * kp:(r + 1) * kp, :], "bf16"))
              for r in range(P)]

    def partials_for(r):
        out = np.zeros((P, mp, N), dtype=np.float32)
        for q in range(P):
            if q != r:
                out[q] = local[q][r * mp:(r + 1) * mp]
        return out
    nothing = np.full((P, mp, N), 0x7FC0, dtype=np.uint16)            # NaN blocks: first pass ignores none of them
    first = [tp_gemm.gemm_ar(P, r, shares[r][0], shares[r][1], "bf16", partials_for(r), nothing) for r in range(P)]
    for r in range(P):
        assert np.array_equal(first[r]["out"], full[r * mp:(r + 1) * mp])
        assert np.array_equal(codec.bf16_decode(first[r]["bcast_bf16"]), full[r * mp:(r + 1) * mp])
        got = codec.bf16_decode(first[r]["full_bf16"])
        assert np.array_equal(got[r * mp:(r + 1) * mp], full[r * mp:(r + 1) * mp])
        others = np.delete(got.reshape(P, mp, N), r, axis=0)
        assert np.isnan(others).all()                                  # received blocks pass through untouched
    handed = np.stack([first[q]["bcast_bf16"] for q in range(P)])
    for r in range(P):
        handed_r = handed.copy()
        handed_r[r] = 0x7FC0                                           # own block must come from the reduction
        res = tp_gemm.gemm_ar(P, r, shares[r][0], shares[r][1], "bf16", partials_for(r), handed_r)
        assert np.array_equal(codec.bf16_decode(res["full_bf16"]), full)


def test_gemm_ar_rounds_own_rows_once_and_checks_shapes():
    P, M, N, K = 2, 4, 8, 128
    g = wl.global_problem(M, N, K, "bf16", seed=9)
    a, b = wl.slice_gemm_rs(g, P, 1)
    partials = np.zeros((P, M // P, N), dtype=np.float32)
    partials[0] = 1.0 + 2.0 ** -9                                      # not a bf16 value
    peer = np.zeros((P, M // P, N), dtype=np.uint16)
    res = tp_gemm.gemm_ar(P, 1, a, b, "bf16", partials, peer)
    rs = tp_gemm.gemm_rs(P, 1, a, b, "bf16", partials)
    assert np.array_equal(res["bcast_bf16"], codec.bf16_encode(rs["out"]))
    assert np.array_equal(res["full_bf16"][M // P:], res["bcast_bf16"])
    assert np.array_equal(res["full_bf16"][:M // P], peer[0])
    with pytest.raises(ValueError):
        tp_gemm.gemm_ar(P, 1, a, b, "bf16", partials, peer.astype(np.float32))
    with pytest.raises(ValueError):
        tp_gemm.gemm_ar(P, 1, a, b, "bf16", partials, peer[:, :1])


def test_bf16_partial_slots_round_every_contribution_once():
    """s = 2 variant: the own contribution is rounded to bf16 before the sum, the peers' slots are bf16.
    Hand-made case: own = 1 + 2^-8 (a tie, rounds to 1.0), peer slot = 2^-8.  bf16 slots: 1.0 + 2^-8 is again a
    tie and ends at 0x3F80; fp32 slots keep own exact: 1 + 2^-7 = 0x3F81."""
    a = codec.bf16_encode(np.array([[1.0, 2.0 ** -8]]))              # 1 x 2
    b = codec.bf16_encode(np.array([[1.0], [1.0]]))                  # 2 x 1
    P, rank = 1, 0
    assert tp_gemm.local_product(a, b, "bf16")[0, 0] == 1.0 + 2.0 ** -8
    # P = 2 with rank 0 owning row 0 (M = 2: second row of A is zero)
    a2 = np.concatenate([a, np.zeros_like(a)], axis=0)
    p32 = np.zeros((2, 1, 1), np.float32)
    p32[1] = 2.0 ** -8
    p16 = codec.bf16_encode(p32.astype(np.float64))
    r32 = tp_gemm.gemm_rs(2, 0, a2, b, "bf16", p32)
    r16 = tp_gemm.gemm_rs(2, 0, a2, b, "bf16", p16, partial_dtype="bf16")
    assert r32["out"][0, 0] == 1.0 + 2.0 ** -7 and r32["out_bf16"][0, 0] == 0x3F81
    assert r16["out"][0, 0] == 1.0 + 2.0 ** -8 and r16["out_bf16"][0, 0] == 0x3F80
    rows32 = tp_gemm.gemm_rs_rows(2, 0, a2, b, "bf16", p32, [0, 1])[1]
    rows16 = tp_gemm.gemm_rs_rows(2, 0, a2, b, "bf16", p16, [0, 1], partial_dtype="bf16")[1]
    assert rows32[0, 0] == r32["out"][0, 0] and rows16[0, 0] == r16["out"][0, 0]
    assert np.isnan(rows16[1]).all()
    with pytest.raises(ValueError):
        tp_gemm.gemm_rs(2, 0, a2, b, "bf16", p32, partial_dtype="bf16")      # float32 array is not bit patterns
    with pytest.raises(ValueError):
        tp_gemm.gemm_rs(2, 0, a2, b, "bf16", p32, partial_dtype="fp16")


@pytest.mark.parametrize("P,M,N,K", [(2, 4, 3, 6), (4, 8, 2, 8)])
def test_bf16_partial_slots_integer_problem_equals_fp32_slots(P, M, N, K):
    """Small integers are exact in bf16, so both slot types give the rows of the unsharded product."""
    A = wl.small_int_matrix((M, K), 41, 1)
    B = wl.small_int_matrix((K, N), 41, 2)
    full = np.array(_brute_int(A, B), dtype=np.float64)
    kp, mp = K // P, M // P
    local = [np.array(_brute_int(A[:, r * kp:(r + 1) * kp], B[r * kp:(r + 1) * kp, :]), dtype=np.float64)
             for r in range(P)]
    for r in range(P):
        p32 = np.zeros((P, mp, N), dtype=np.float32)
        for q in range(P):
            if q != r:
                p32[q] = local[q][r * mp:(r + 1) * mp]
        p16 = codec.bf16_encode(p32.astype(np.float64))
        a, b = _int_bits(A[:, r * kp:(r + 1) * kp], "bf16"), _int_bits(B[r * kp:(r + 1) * kp, :], "bf16")
        res = tp_gemm.gemm_rs(P, r, a, b, "bf16", p16, partial_dtype="bf16")
        assert np.array_equal(res["out"], full[r * mp:(r + 1) * mp])
        peer = np.zeros((P, mp, N), np.uint16)
        ar = tp_gemm.gemm_ar(P, r, a, b, "bf16", p16, peer, partial_dtype="bf16")
        assert np.array_equal(codec.bf16_decode(ar["bcast_bf16"]), full[r * mp:(r + 1) * mp])


@pytest.mark.parametrize("P,M,N,K", [(2, 3, 4, 6), (3, 5, 6, 9), (4, 2, 8, 8)])
def test_gemm_rs_cols_integer_brute_force_all_ranks(P, M, N, K):
    """Last-dimension scatter on one global integer problem with true partials: rank r ends with the column block
    N_r of the unsharded product, the blocks side by side give the whole product, and slot q of `outgoing` is the
    column block N_q of the local product."""
    A = wl.small_int_matrix((M, K), 61, 1)
    B = wl.small_int_matrix((K, N), 61, 2)
    full = np.array(_brute_int(A, B), dtype=np.float64)
    kp, np_ = K // P, N // P
    local = [np.array(_brute_int(A[:, r * kp:(r + 1) * kp], B[r * kp:(r + 1) * kp, :]), dtype=np.float64)
             for r in range(P)]
    blocks = []
    for r in range(P):
        partials = np.zeros((P, M, np_), dtype=np.float32)
        for q in range(P):
            if q != r:
                partials[q] = local[q][:, r * np_:(r + 1) * np_]
        partials[r] = -777.0                                      # must be ignored
        res = tp_gemm.gemm_rs_cols(P, r, _int_bits(A[:, r * kp:(r + 1) * kp], "bf16"),
                                   _int_bits(B[r * kp:(r + 1) * kp, :], "bf16"), "bf16", partials)
        assert np.array_equal(res["own"], local[r])
        for q in range(P):
            assert np.array_equal(res["outgoing"][q], local[r][:, q * np_:(q + 1) * np_])
        assert np.array_equal(res["out"], full[:, r * np_:(r + 1) * np_])
        blocks.append(codec.bf16_decode(res["out_bf16"]))
    assert np.array_equal(np.concatenate(blocks, axis=1), full)
    with pytest.raises(ValueError):
        tp_gemm.gemm_rs_cols(P, 0, _int_bits(A[:, :kp], "bf16"), _int_bits(B[:kp, :], "bf16"), "bf16",
                             np.zeros((P, M, np_ + 1), np.float32))


def test_gather_along_the_last_dimension():
    """Column chunk q holds columns K_q; the product with the column-gathered A equals the sum over chunks of
    chunk_q . B[K_q, :] (integers: exactly), whatever the order the chunks are combined in."""
    P, M, N, K = 3, 4, 5, 9
    A = wl.small_int_matrix((M, K), 71, 1)
    B = wl.small_int_matrix((K, N), 71, 2)
    kp = K // P
    chunks = [_int_bits(A[:, q * kp:(q + 1) * kp], "bf16") for q in range(P)]
    G = tp_gemm.gather_kchunks(chunks)
    assert G.shape == (M, K)
    for q in range(P):
        assert np.array_equal(G[:, q * kp:(q + 1) * kp], chunks[q])
    full = np.array(_brute_int(A, B), dtype=np.float64)
    got = tp_gemm.ag_gemm(P, 1, G, _int_bits(B, "bf16"), "bf16")["C"] if M % P == 0 else \
        tp_gemm.local_product(G, _int_bits(B, "bf16"), "bf16")
    assert np.array_equal(got, full)
    by_chunk = sum(np.array(_brute_int(A[:, q * kp:(q + 1) * kp], B[q * kp:(q + 1) * kp, :]), dtype=np.float64)
                   for q in (2, 0, 1))
    assert np.array_equal(by_chunk, full)


def test_activation_closed_forms_and_identities():
    x = np.linspace(-6, 6, 97)
    for kind in ("silu", "gelu_tanh"):
        y = tp_gemm.activation(x, kind)
        assert np.allclose(y - tp_gemm.activation(-x, kind), x, rtol=0, atol=1e-15)      # f(x) - f(-x) = x
        assert tp_gemm.activation(0.0, kind) == 0.0
        assert np.all(np.diff(y[x >= 0]) > 0)                                            # increasing on x >= 0
        assert abs(tp_gemm.activation(30.0, kind) - 30.0) < 1e-9 and abs(tp_gemm.activation(-30.0, kind)) < 1e-9
    assert abs(tp_gemm.activation(1.0, "silu") - 0.7310585786300049) < 1e-15             # 1 / (1 + e^-1)
    assert abs(tp_gemm.activation(1.0, "gelu_tanh") - 0.8411919906082768) < 1e-12        # published value of the tanh form
    # the tanh form stays within 5e-4 of x * Phi(x) (standard normal distribution function)
    from math import erf, sqrt
    exact = np.array([v * 0.5 * (1.0 + erf(v / sqrt(2.0))) for v in x])
    assert np.max(np.abs(tp_gemm.activation(x, "gelu_tanh") - exact)) < 5e-4
    assert np.array_equal(tp_gemm.activation(np.array([-2.0, 0.0, 3.0]), "relu"), [0.0, 0.0, 3.0])
    assert np.array_equal(tp_gemm.activation(x, "none"), x) and np.array_equal(tp_gemm.activation(x, None), x)
    with pytest.raises(ValueError):
        tp_gemm.activation(x, "tanh")


def test_mlp_block_chains_the_two_ops_through_bf16():
    """Integer problem with relu: H and the output are exact, so the chain can be brute-forced."""
    P, M, I, D = 2, 4, 6, 3                    # X: M x D gathered, W1: D x I, W2: I x D
    X = wl.small_int_matrix((M, D), 51, 1)
    W1 = wl.small_int_matrix((D, I), 51, 2)
    W2 = wl.small_int_matrix((I, D), 51, 3)
    ip, mp = I // P, M // P
    H = [[max(v, 0) for v in row] for row in _brute_int(X, W1)]                            # relu, integers
    full = np.array(_brute_int(np.array(H, dtype=np.float32), W2), dtype=np.float64)
    for r in range(P):
        cols = slice(r * ip, (r + 1) * ip)
        partials = np.zeros((P, mp, D), np.float32)
        for q in range(P):
            if q != r:
                cq = slice(q * ip, (q + 1) * ip)
                hq = np.array(H, dtype=np.float32)[:, cq]
                partials[q] = np.array(_brute_int(hq, W2[cq, :]), dtype=np.float32)[r * mp:(r + 1) * mp]
        res = tp_gemm.mlp_block(P, r, _int_bits(X, "bf16"), _int_bits(W1[:, cols], "bf16"), _int_bits(W2[cols, :], "bf16"),
                                partials, act="relu")
        assert np.array_equal(codec.bf16_decode(res["H_bf16"]), np.array(H, dtype=np.float64)[:, cols])
        assert np.array_equal(res["out"], full[r * mp:(r + 1) * mp])
    # H is rounded to bf16 before the second GEMM: 1 + 2^-8 (a tie) becomes 1.0
    x = codec.bf16_encode(np.array([[1.0, 2.0 ** -8]]))
    w1 = codec.bf16_encode(np.array([[1.0], [1.0]]))
    w2 = codec.bf16_encode(np.array([[1.0]]))
    res = tp_gemm.mlp_block(1, 0, x, w1, w2, np.zeros((1, 1, 1), np.float32), act="none")
    assert res["H_bf16"][0, 0] == 0x3F80 and res["out"][0, 0] == 1.0


def test_linearity_and_shard_concatenation_random_bf16():
    """Sum over ranks of A[:,K_p].B[K_p,:] equals the unsharded GEMM (to float64 rounding),
    and the P reduced shards stacked give the whole product."""
    P, M, N, K = 4, 16, 12, 64
    g = wl.global_problem(M, N, K, "bf16", seed=3)
    A = codec.bf16_decode(g["A"])
    B = codec.bf16_decode(g["B"])
    full = np.zeros((M, N))
    for i in range(M):                        # independent plain evaluation, k ascending
        for j in range(N):
            s = 0.0
            for t in range(K):
                s += A[i, t] * B[t, j]
            full[i, j] = s
    mp = M // P
    shares = [wl.slice_gemm_rs(g, P, r) for r in range(P)]
    owns = [tp_gemm.local_product(a, b, "bf16") for a, b in shares]
    assert np.allclose(sum(owns), full, rtol=0, atol=K * 2.0 ** -52)
    shards = []
    for r in range(P):
        partials = np.zeros((P, mp, N), dtype=np.float32)
        for q in range(P):
            if q != r:
                partials[q] = owns[q][r * mp:(r + 1) * mp].astype(np.float32)
        shards.append(tp_gemm.gemm_rs(P, r, shares[r][0], shares[r][1], "bf16", partials)["out"])
    stacked = np.concatenate(shards, axis=0)
    # peers' contributions were rounded to float32 on the way: 3 roundings of ~|x|*2^-24 each
    assert np.allclose(stacked, full, rtol=0, atol=4 * 2.0 ** -24)


def test_ag_gemm_concatenation_and_chunk_order():
    P, M, N, K = 4, 8, 12, 10
    A = wl.small_int_matrix((M, K), 31, 1)
    B = wl.small_int_matrix((K, N), 31, 2)
    full = np.array(_brute_int(A, B), dtype=np.float64)
    g = {"A": _int_bits(A, "bf16"), "B": _int_bits(B, "bf16")}
    chunks = [wl.slice_ag_gemm(g, P, q)[0] for q in range(P)]
    gathered = tp_gemm.gather_chunks(chunks)
    assert np.array_equal(gathered, g["A"])                       # A_gathered == concat of the chunks
    cols = []
    for r in range(P):
        _, b_loc = wl.slice_ag_gemm(g, P, r)
        res = tp_gemm.ag_gemm(P, r, gathered, b_loc, "bf16")
        assert res["C"].shape == (M, N // P)
        cols.append(res["C"])
    assert np.array_equal(np.concatenate(cols, axis=1), full)
    sub = tp_gemm.ag_gemm(P, 1, gathered, wl.slice_ag_gemm(g, P, 1)[1], "bf16", rows=[5, 0])
    assert np.array_equal(sub["C"], full[[5, 0], 3:6])


def test_reduce_closed_forms():
    P, mp, N = 5, 3, 4
    consts = np.array([1.5, -2.25, 4.0, 0.125, 7.0], dtype=np.float32)
    partials = np.broadcast_to(consts[:, None, None], (P, mp, N)).copy()
    assert np.array_equal(tp_gemm.reduce_partials(partials), np.full((mp, N), consts.astype(np.float64).sum()))
    x = np.random.default_rng(2).standard_normal((mp, N)).astype(np.float32)
    pm = np.stack([x, -x, 2 * x, -2 * x])
    assert np.array_equal(tp_gemm.reduce_partials(pm), np.zeros((mp, N)))
    assert np.array_equal(tp_gemm.reduce_partials(x[None]), x.astype(np.float64))
    # sums that float32 would get wrong but float64 keeps: 2^24 + 1 - 2^24 = 1
    big = np.stack([np.full((1, 1), 2.0 ** 24, np.float32), np.ones((1, 1), np.float32),
                    np.full((1, 1), -2.0 ** 24, np.float32)])
    assert tp_gemm.reduce_partials(big)[0, 0] == 1.0


def test_gemm_rs_P1_is_plain_rounded_gemm():
    A = wl.small_int_matrix((4, 6), 41, 1)
    B = wl.small_int_matrix((6, 3), 41, 2)
    res = tp_gemm.gemm_rs(1, 0, _int_bits(A, "bf16"), _int_bits(B, "bf16"), "bf16",
                          np.zeros((1, 4, 3), np.float32))
    assert np.array_equal(res["out"], np.array(_brute_int(A, B), dtype=np.float64))


def test_rows_variants_agree_with_definitions():
    P, M, N, K = 2, 8, 5, 12
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank=1, seed=4)
    A = codec.bf16_decode(inp["A_local"])
    B = codec.bf16_decode(inp["B_local"])
    rows = [7, 0, 4, 3]
    own_rows, out_rows = tp_gemm.gemm_rs_rows(P, 1, inp["A_local"], inp["B_local"], "bf16", inp["partials"], rows)
    for t, i in enumerate(rows):
        for j in range(N):
            ref = sum(A[i, k] * B[k, j] for k in range(K // P))
            assert abs(own_rows[t, j] - ref) <= 1e-15
            if i >= 4:
                red = float(inp["partials"][0][i - 4, j]) + ref
                assert abs(out_rows[t, j] - red) <= 1e-15
            else:
                assert np.isnan(out_rows[t, j])


def test_abs_product_bounds_the_sum():
    inp = wl.gemm_rs_inputs(2, 8, 6, 16, "bf16", rank=0, seed=5)
    own = tp_gemm.local_product(inp["A_local"], inp["B_local"], "bf16")
    mag = tp_gemm.abs_product(inp["A_local"], inp["B_local"], "bf16")
    assert np.all(np.abs(own) <= mag + 1e-18)
    assert np.all(mag > 0)


def test_abs_product_equals_an_integer_sum_of_magnitudes():
    """Pin of the bound helper: on small-integer operands sum_k |a_ik| |b_kj| is exact in Python integers (a factor,
    a dropped absolute value or a transposed operand would show), and an fp8 scale pair enters once, in magnitude."""
    rng = np.random.default_rng(11)
    for (m, k, n) in ((3, 5, 4), (7, 13, 2), (1, 1, 1)):
        ia = rng.integers(-3, 4, size=(m, k))
        ib = rng.integers(-3, 4, size=(k, n))
        a_bits = codec.bf16_encode(ia.astype(np.float64))
        b_bits = codec.bf16_encode(ib.astype(np.float64))
        want = [[sum(abs(int(ia[i, t])) * abs(int(ib[t, j])) for t in range(k)) for j in range(n)] for i in range(m)]
        got = tp_gemm.abs_product(a_bits, b_bits, "bf16")
        assert got.shape == (m, n)
        assert np.array_equal(got, np.array(want, dtype=np.float64))
        assert np.array_equal(tp_gemm.abs_product(a_bits, b_bits, "bf16", rows=[m - 1]), np.array(want, dtype=np.float64)[m - 1:])
    # e4m3: codes 0x38 = 1, 0x40 = 2, 0xC0 = -2; scales 0.5 and -3 -> |scale| = 1.5
    a8 = np.array([[0x38, 0xC0], [0x40, 0x40]], dtype=np.uint8)
    b8 = np.array([[0xC0], [0x38]], dtype=np.uint8)
    got = tp_gemm.abs_product(a8, b8, "fp8", 0.5, -3.0)
    assert np.array_equal(got, 1.5 * np.array([[1 * 2 + 2 * 1], [2 * 2 + 2 * 1]], dtype=np.float64))


def test_shape_errors():
    a = np.zeros((4, 6), np.uint16)
    with pytest.raises(ValueError):
        tp_gemm.local_product(a, np.zeros((5, 3), np.uint16), "bf16")
    with pytest.raises(ValueError):
        tp_gemm.gemm_rs(3, 0, a, np.zeros((6, 3), np.uint16), "bf16", np.zeros((3, 1, 3), np.float32))
    with pytest.raises(ValueError):
        tp_gemm.gemm_rs(2, 0, a, np.zeros((6, 3), np.uint16), "bf16", np.zeros((2, 2, 4), np.float32))
