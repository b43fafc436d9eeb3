"""GPU parity on hand-placed special values: bf16 subnormals, signed zeros, infinities, NaN, sums that overflow the
output format, e4m3 subnormal codes.  The oracle keeps NaN, does not flush subnormals and rounds once; these tests
compare that reading with what the MFMA and the conversion instructions do.  NaN: positions are compared (the payload
and sign of a NaN are not part of the contract); infinities must match exactly; finite elements by the usual gate."""
import numpy as np
import pytest

from oracle import codec, tp_gemm
from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu

GATE = {"bf16": 1e-2, "fp8": 5e-2}


def compare(got, ref, dtype):
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan), "NaN positions differ"
    inf = np.isinf(ref)
    assert np.array_equal(got[inf], ref[inf]), "infinities differ"
    fin = ~nan & ~inf
    # after rounding to bf16 the result may be infinite where the unrounded reference is finite: compare with the rounded one
    rb = codec.bf16_decode(codec.bf16_encode(np.where(fin, ref, 0.0)))
    both_fin = fin & np.isfinite(rb)
    assert np.array_equal(np.isinf(got[fin]), np.isinf(rb[fin])), "overflow to infinity differs"
    assert np.array_equal(got[fin & np.isinf(rb)], rb[fin & np.isinf(rb)])
    err = np.abs(got[both_fin] - ref[both_fin]) / (np.abs(ref[both_fin]) + 1.0)
    assert err.size == 0 or float(err.max()) <= GATE[dtype]
    return rb


def planted_bf16(M, N, K, seed):
    """A and B: rows 0..15 of A are zero except planted entries, the rest is the usual N(0,1)/sqrt(K) data."""
    inp = wl.ag_gemm_inputs(1, M, N, K, "bf16", 0, seed=seed)
    A = np.array(inp["chunks"][0], dtype=np.uint16)
    B = np.array(inp["B_local"], dtype=np.uint16)
    A[:16] = 0
    B[0, :16] = 0x3F80                         # 1.0 in the first k-row of the first 16 columns
    A[0, 0] = 0x0001                           # smallest subnormal, 2^-133
    B[0, 0] = 0x7180                           # 2^100: the product 2^-33 is normal
    A[1, 0] = 0x0040                           # subnormal 2^-127 times 1.0: a subnormal result
    A[2, 0] = 0x0080                           # smallest normal times 0.5: result below the normal range
    B[0, 2] = 0x3F00
    A[3, 0] = 0x8000                           # -0
    A[4, 0] = 0x7FC0                           # NaN: the whole output row
    A[5, 0] = 0x7F80                           # +inf
    A[6, 0] = 0xFF80                           # -inf
    A[7, 0] = 0x7F7F                           # largest finite, doubled: overflows in the accumulator
    B[0, 7] = 0x4000
    A[8, 0] = 0x7F7F                           # largest finite times (1 + 2^-7): finite in fp32, rounds to bf16 infinity
    A[8, 1] = 0x7F7F
    B[0, 8] = 0x3F80
    B[1, 8] = 0x3C00
    A[9, 0] = 0x807F                           # largest negative subnormal
    A[10, :] = 0x0001                          # a row of subnormals against ordinary B columns
    return A, B


@pytest.mark.parametrize("M,N,K", [(384, 264, 128), (4096, 4096, 64)])   # the 128 x 128 and the 256 x 256 kernels
def test_ag_gemm_bf16_special_values(M, N, K):
    A, B = planted_bf16(M, N, K, seed=51)
    assert pk.pk_ag_gemm_plan(1, M, N, K, "bf16").tile_m == (128 if M < 4096 else 256)
    res = hz.run_ag_gemm(1, 0, M, N, K, "bf16", [A], B)
    assert res["status"][0] == 0
    with np.errstate(invalid="ignore", over="ignore"):
        ref = tp_gemm.ag_gemm(1, 0, A, B, "bf16")["C"]
    got = codec.bf16_decode(res["C_bits"])
    rb = compare(got, ref, "bf16")
    # the planted results exactly: subnormal products and results are kept, not flushed
    bits = res["C_bits"]
    assert bits[0, 0] == 0x2F00                # 2^-33
    assert bits[1, 1] == 0x0040                # 2^-127
    assert bits[2, 2] == 0x0040                # 2^-126 * 0.5
    assert bits[3, 3] in (0x0000, 0x8000)      # a zero; its sign depends on the accumulator's starting zero
    assert bits[5, 5] == 0x7F80 and bits[6, 6] == 0xFF80
    assert bits[7, 7] == 0x7F80 and bits[8, 8] == 0x7F80
    assert bits[9, 9] == 0x807F
    assert np.array_equal(got[10], rb[10]) or np.max(np.abs(got[10] - ref[10])) <= 2.0 ** -125


def test_ag_gemm_fp8_subnormal_codes_and_nan():
    """Planted e4m3 codes in otherwise zero operands, scales 1: every product and sum here is exact in fp32."""
    M, N, K = 384, 272, 256
    A = np.zeros((M, K), dtype=np.uint8)
    B = np.zeros((K, N), dtype=np.uint8)
    B[0, :8] = 0x38                            # 1.0
    A[0, 0] = 0x01                             # 2^-9, the smallest e4m3 subnormal
    A[1, 0] = 0x07                             # 7 * 2^-9 times itself
    B[0, 1] = 0x07
    A[2, 0] = 0x7F                             # NaN
    A[3, 0] = 0x7E                             # 448 * 448
    B[0, 3] = 0x7E
    A[4, 0] = 0x81                             # -2^-9 * 2^-9
    B[0, 4] = 0x01
    A[5, :] = 0x01                             # a row of the smallest subnormal against columns of small codes
    B[:, 8:] = (np.arange(K * (N - 8)).reshape(K, N - 8) % 5).astype(np.uint8)
    res = hz.run_ag_gemm(1, 0, M, N, K, "fp8", [A], B, scale_a=1.0, scale_b=1.0)
    assert res["status"][0] == 0
    with np.errstate(invalid="ignore"):
        ref = tp_gemm.ag_gemm(1, 0, A, B, "fp8", 1.0, 1.0)["C"]
    got = codec.bf16_decode(res["C_bits"])
    rb = compare(got, ref, "fp8")
    bits = res["C_bits"]
    assert bits[0, 0] == 0x3B00 and bits[1, 1] == 0x3944 and bits[3, 3] == 0x4844 and bits[4, 4] == 0xB680
    assert np.array_equal(got[5], rb[5])       # sums of subnormal products: exact, then rounded once


def test_gemm_rs_special_partials():
    """Peer partials with a NaN, infinities, sums that round to bf16 infinity, subnormals; own contribution zero there."""
    P, rank, M, N, K = 2, 0, 512, 384, 256
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=53)
    A = np.array(inp["A_local"], dtype=np.uint16)
    A[:8] = 0                                  # own product is zero in the first rows of the own shard
    part = np.array(inp["partials"], dtype=np.float32)
    part[1, :8] = 0.0
    part[1, 0, 0] = np.nan
    part[1, 1, 1] = np.inf
    part[1, 2, 2] = -np.inf
    part[1, 3, 3] = np.float32(3.4e38)         # finite in fp32, above the largest bf16: rounds to infinity
    part[1, 4, 4] = np.float32(2.0 ** -149)    # smallest fp32 subnormal: rounds to zero in bf16
    part[1, 5, 5] = np.float32(2.0 ** -133)    # smallest bf16 subnormal survives
    part[1, 6, 6] = np.float32(-0.0)
    res = hz.run_gemm_rs(P, rank, M, N, K, "bf16", A, inp["B_local"], part)
    assert res["status"][0] == 0
    with np.errstate(invalid="ignore", over="ignore"):
        ref = tp_gemm.gemm_rs(P, rank, A, inp["B_local"], "bf16", part)
    got = codec.bf16_decode(res["out_bits"])
    compare(got, ref["out"], "bf16")
    bits = res["out_bits"]
    assert bits[1, 1] == 0x7F80 and bits[2, 2] == 0xFF80 and bits[3, 3] == 0x7F80
    assert bits[4, 4] in (0x0000, 0x8000) and bits[5, 5] == 0x0001
