"""Seeded synthetic workloads for the two tensor-parallel ops.

This module only draws random numbers, rounds them to the storage formats with
library conversions, and slices buffers.  It holds none of the arithmetic of
the method (no GEMM, no reduction) and imports neither the HIP binding nor the
CPU oracle; the tests and the benchmark feed its outputs to both.

The paper measures on synthetic GEMMs of local shape N x N x N/8 (GEMM+RS) and
N x N/8 x N (AG+GEMM) on 8 ranks (section 4.1); the configurations here are of
that family, at the shapes of a 70B-class MLP under 8-way tensor parallelism
for the two large bf16 cases.  All dimensions below are GLOBAL (M, N, K of the
unsharded GEMM), as in the paper's notation.
"""
from dataclasses import dataclass

import numpy as np
import torch

BASE_SEED = 251113940


@dataclass(frozen=True)
class Config:
    name: str
    op: str          # "gemm_rs" or "ag_gemm"
    P: int
    M: int
    N: int
    K: int
    dtype: str       # "bf16" or "fp8"
    order: str       # arrival order of the peers' data: "random" or "ring"

    @property
    def local_mnk(self):
        if self.op == "gemm_rs":
            return self.M, self.N, self.K // self.P
        return self.M, self.N // self.P, self.K

    @property
    def flops(self):
        m, n, k = self.local_mnk
        return 2 * m * n * k


CONFIGS = {
    # local 256x256x256, one peer partial of 128x256
    "cfg1": Config("cfg1", "gemm_rs", 2, 256, 256, 512, "bf16", "random"),
    # A gathered from 4 chunks of 512x2048, B_local 2048x1024
    "cfg2": Config("cfg2", "ag_gemm", 4, 2048, 4096, 2048, "bf16", "random"),
    # 70B MLP down-projection share: A_local 8192x3584, B_local 3584x8192
    "cfg3": Config("cfg3", "gemm_rs", 8, 8192, 8192, 28672, "bf16", "ring"),
    # 70B MLP up-projection share: A 8192x8192 from 8 chunks, B_local 8192x3584
    "cfg4": Config("cfg4", "ag_gemm", 8, 8192, 28672, 8192, "bf16", "ring"),
    # fp8 e4m3 inputs with per-tensor scales: A_local 16384x2048, B_local 2048x16384
    "cfg5": Config("cfg5", "gemm_rs", 8, 16384, 16384, 16384, "fp8", "ring"),
}


def _rng(seed, stream):
    return np.random.default_rng([BASE_SEED, int(seed), int(stream)])


def _normal(rng, shape, sigma):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(sigma)
    return x


def to_bf16_bits(x_f32):
    """float32 array -> uint16 bf16 bit patterns (library round-to-nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def to_fp8_bits(x_f32):
    """float32 array -> (uint8 e4m3 bit patterns, float32 per-tensor scale).

    scale = amax/448; the stored code is the library's nearest-even e4m3 of
    x/scale, clamped to the finite range first (the library cast does not
    saturate).
    """
    amax = float(np.max(np.abs(x_f32))) if x_f32.size else 0.0
    scale = np.float32(amax / 448.0) if amax > 0 else np.float32(1.0)
    y = torch.from_numpy(np.ascontiguousarray(x_f32)) / float(scale)
    y = y.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn)
    return y.view(torch.uint8).numpy(), scale


def _quantise(x_f32, dtype):
    if dtype == "bf16":
        return to_bf16_bits(x_f32), None
    if dtype == "fp8":
        return to_fp8_bits(x_f32)
    raise ValueError(dtype)


def arrival_order(P, rank, kind, seed=0):
    """The order in which the P-1 peers' data lands (own data is present at call).

    "ring":   rank+1, rank+2, ... (mod P);  "random": a seeded permutation.
    """
    peers = [(rank + d) % P for d in range(1, P)]
    if kind == "ring":
        return peers
    if kind == "random":
        perm = _rng(seed, 900 + rank).permutation(len(peers))
        return [peers[i] for i in perm]
    raise ValueError(kind)


def gemm_rs_inputs(P, M, N, K, dtype, rank, seed=0, order="ring"):
    """Inputs of one rank of GEMM+RS with i.i.d. synthetic peer partials.

    A_local (M x K/P) and B_local (K/P x N) are z/sqrt(K), z ~ N(0,1), rounded
    to the storage format.  Peer partial slots are float32 N(0, sigma_p^2) with
    sigma_p = sqrt(K/P)/K, the standard deviation of a true partial sum under
    this input distribution.  Slot `rank` is zero (the op writes it).
    """
    kp, mp = K // P, M // P
    sig = 1.0 / np.sqrt(K)
    a_bits, sa = _quantise(_normal(_rng(seed, 1 + rank), (M, kp), sig), dtype)
    b_bits, sb = _quantise(_normal(_rng(seed, 101 + rank), (kp, N), sig), dtype)
    partials = np.zeros((P, mp, N), dtype=np.float32)
    sig_p = np.sqrt(kp) / K
    for q in range(P):
        if q != rank:
            partials[q] = _normal(_rng(seed, 201 + rank * 64 + q), (mp, N), sig_p)
    return {"A_local": a_bits, "B_local": b_bits, "scale_a": sa, "scale_b": sb,
            "partials": partials, "order": arrival_order(P, rank, order, seed)}


def global_problem(M, N, K, dtype, seed=0):
    """A seeded GLOBAL problem (A: M x K, B: K x N) from which every rank's share can be sliced."""
    sig = 1.0 / np.sqrt(K)
    a_bits, sa = _quantise(_normal(_rng(seed, 301), (M, K), sig), dtype)
    b_bits, sb = _quantise(_normal(_rng(seed, 302), (K, N), sig), dtype)
    return {"A": a_bits, "B": b_bits, "scale_a": sa, "scale_b": sb}


def slice_gemm_rs(g, P, rank):
    """Rank's share of a global problem for GEMM+RS: A[:, K_r], B[K_r, :]."""
    K = g["A"].shape[1]
    kp = K // P
    ks = slice(rank * kp, (rank + 1) * kp)
    return np.ascontiguousarray(g["A"][:, ks]), np.ascontiguousarray(g["B"][ks, :])


def slice_ag_gemm(g, P, rank):
    """Rank's share of a global problem for AG+GEMM: chunk r of A, B[:, N_r]."""
    M, N = g["A"].shape[0], g["B"].shape[1]
    mp, np_ = M // P, N // P
    return (np.ascontiguousarray(g["A"][rank * mp:(rank + 1) * mp]),
            np.ascontiguousarray(g["B"][:, rank * np_:(rank + 1) * np_]))


def ag_gemm_inputs(P, M, N, K, dtype, rank, seed=0, order="ring"):
    """Inputs of one rank of AG+GEMM: the P row-chunks of A (chunk q "arrives"
    from rank q) and B_local = B[:, N_rank] (K x N/P)."""
    mp, np_ = M // P, N // P
    sig = 1.0 / np.sqrt(K)
    if dtype == "fp8":
        # one scale for the whole gathered operand, so every chunk dequantises alike
        a_all, sa = _quantise(_normal(_rng(seed, 401), (M, K), sig), dtype)
        chunks = [np.ascontiguousarray(a_all[q * mp:(q + 1) * mp]) for q in range(P)]
    else:
        chunks, sa = [], None
        for q in range(P):
            cb, _ = _quantise(_normal(_rng(seed, 401 + q), (mp, K), sig), dtype)
            chunks.append(cb)
    b_bits, sb = _quantise(_normal(_rng(seed, 501 + rank), (K, np_), sig), dtype)
    return {"chunks": chunks, "B_local": b_bits, "scale_a": sa, "scale_b": sb,
            "order": arrival_order(P, rank, order, seed)}


def small_int_matrix(shape, seed, stream, lo=-2, hi=2):
    """Integer-valued float32 matrix with entries in [lo, hi] (exactly representable everywhere)."""
    return _rng(seed, stream).integers(lo, hi + 1, size=shape).astype(np.float32)
