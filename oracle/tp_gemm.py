"""Plain definitions of the two tensor-parallel results, in float64.

Test infrastructure only (see the package docstring).

Notation follows the paper (section 4, experimental setup; figures "AG + GEMM"
and "GEMM + RS"): P ranks, a global GEMM M x N x K with A of shape M x K and B
of shape K x N, both row-major.

GEMM + reduce-scatter (sections 3.1.3 and 4.1).  Rank r holds the K-slice
K_r = [r*K/P, (r+1)*K/P): A_local = A[:, K_r] (M x K/P) and B_local = B[K_r, :]
(K/P x N).  Its local product own = A_local . B_local is a full M x N matrix of
partial sums; the rows R_q = [q*M/P, (q+1)*M/P) of it belong to rank q.  The
result rank r ends up with is its shard of the reduced matrix,
    out[i', j] = sum_{p<P} (A[:, K_p] . B[K_p, :])[r*M/P + i', j].
The method only overlaps the exchange with the GEMM; it reaches exactly this
sum (up to rounding order), so the oracle is the sum written out.

All-gather + GEMM (section 4.1).  Rank r holds row-chunk r of A (M/P x K) and
the column slice B[:, N_r] (K x N/P); after the gather it computes
    C[:, N_r] = A . B[:, N_r]                       (M x N/P).
The order in which chunks arrive does not enter the definition.

GEMM + all-reduce (section 3.1.3, inter-SM overlapping; section 4.1, figure
"GEMM + AR").  Same operands as GEMM + reduce-scatter, but every rank ends with
the whole reduced matrix, rounded to bf16:
    full[i, j] = bf16( sum_{p<P} (A[:, K_p] . B[K_p, :])[i, j] )   (M x N).
Rank r reduces the rows R_r (exactly the reduce-scatter result above), rounds
them once and hands that rounded block to every rank; the rows R_q, q != r, of
its own copy are the blocks the other ranks hand to it, taken as they come.

Readings where the paper is silent (the 8-bit path is an extension):
  * the scattered output dimension is the row dimension M;
  * cross-rank sums are taken over per-source partial slots, float32 by
    default, bf16 as the paper's variant (the oracle adds them in float64, slot
    order 0..P-1);
  * 8-bit inputs carry one float32 scale per tensor; the unscaled products are
    accumulated and the product of the two scales is applied once at the end.
"""
import numpy as np

from . import codec


def _scale(scale_a, scale_b):
    sa = 1.0 if scale_a is None else float(np.float32(scale_a))
    sb = 1.0 if scale_b is None else float(np.float32(scale_b))
    return sa * sb


def local_product(a_bits, b_bits, dtype, scale_a=None, scale_b=None, rows=None):
    """(scale_a*scale_b) * A . B in float64 from the stored bit patterns.

    a_bits: m x k, b_bits: k x n.  rows (optional index array) restricts the
    result to those rows of A: the returned array is len(rows) x n.
    """
    a_bits = np.asarray(a_bits)
    b_bits = np.asarray(b_bits)
    if a_bits.ndim != 2 or b_bits.ndim != 2 or a_bits.shape[1] != b_bits.shape[0]:
        raise ValueError(f"shape mismatch {a_bits.shape} x {b_bits.shape}")
    if rows is not None:
        a_bits = a_bits[np.asarray(rows, dtype=np.int64)]
    a = codec.decode(a_bits, dtype)
    b = codec.decode(b_bits, dtype)
    return _scale(scale_a, scale_b) * (a @ b)


def _slot_values(partials, partial_dtype, shape):
    """The partial slots as float64, from float32 values or bf16 bit patterns."""
    partials = np.asarray(partials)
    if partials.shape != shape:
        raise ValueError(f"partials shape {partials.shape} != {shape}")
    if partial_dtype == "f32":
        return partials.astype(np.float64)
    if partial_dtype == "bf16":
        if partials.dtype != np.uint16:
            raise ValueError("bf16 partial slots are passed as uint16 bit patterns")
        return codec.bf16_decode(partials)
    raise ValueError(f"unknown partial dtype {partial_dtype!r}")


def gemm_rs(P, rank, a_local_bits, b_local_bits, dtype, partials,
            scale_a=None, scale_b=None, partial_dtype="f32"):
    """One rank's GEMM + reduce-scatter.

    partial_dtype "f32" (default): the slots hold float32 values.  "bf16": the
    slots hold bf16 values (the paper's element size for communicated tiles,
    section 3.1.3, s = 2), passed as uint16 bit patterns; every contribution,
    this rank's own included, is rounded to bf16 once before the sum.

    a_local_bits: M x K/P, b_local_bits: K/P x N.
    partials:     [P][M/P][N] float32; slot q (q != rank) is what rank q sent for
                  this rank's shard.  Slot `rank` is ignored.
    Returns a dict:
      own       M x N float64, this rank's local product;
      outgoing  [P][M/P][N] float64, slot q = rows R_q of own (what is sent to
                rank q; slot `rank` is this rank's own contribution);
      out       M/P x N float64, the reduced shard, not rounded;
      out_bf16  the same rounded once to bf16 (as uint16 bit patterns).
    """
    own = local_product(a_local_bits, b_local_bits, dtype, scale_a, scale_b)
    M, N = own.shape
    if M % P:
        raise ValueError("M must be a multiple of P")
    mp = M // P
    slots = _slot_values(partials, partial_dtype, (P, mp, N))
    outgoing = own.reshape(P, mp, N)
    mine = outgoing[rank] if partial_dtype == "f32" else codec.bf16_round(outgoing[rank])
    out = np.zeros((mp, N), dtype=np.float64)
    for p in range(P):
        out += mine if p == rank else slots[p]
    return {"own": own, "outgoing": outgoing, "out": out,
            "out_bf16": codec.bf16_encode(out)}


def gemm_rs_cols(P, rank, a_local_bits, b_local_bits, dtype, partials,
                 scale_a=None, scale_b=None, partial_dtype="f32"):
    """GEMM + reduce-scatter along the LAST dimension (appendix "Additional
    collective performance": reduce-scatter along the tensor dimension, whose
    pieces are not contiguous in memory).  Same operands as gemm_rs; rank q owns
    the column block N_q = [q*N/P, (q+1)*N/P) of every row:
        out[i, j'] = sum_{p<P} (A[:, K_p] . B[K_p, :])[i, rank*N/P + j']      (M x N/P).
    partials: [P][M][N/P]; slot q != rank is what rank q sent, slot `rank` ignored.
    Returns own (M x N), outgoing ([P][M][N/P]: slot q = columns N_q of own),
    out (M x N/P float64), out_bf16.
    """
    own = local_product(a_local_bits, b_local_bits, dtype, scale_a, scale_b)
    M, N = own.shape
    if N % P:
        raise ValueError("N must be a multiple of P")
    np_ = N // P
    slots = _slot_values(partials, partial_dtype, (P, M, np_))
    outgoing = np.stack([own[:, q * np_:(q + 1) * np_] for q in range(P)])
    mine = outgoing[rank] if partial_dtype == "f32" else codec.bf16_round(outgoing[rank])
    out = np.zeros((M, np_), dtype=np.float64)
    for p in range(P):
        out += mine if p == rank else slots[p]
    return {"own": own, "outgoing": outgoing, "out": out,
            "out_bf16": codec.bf16_encode(out)}


def gemm_rs_rows(P, rank, a_local_bits, b_local_bits, dtype, partials, rows,
                 scale_a=None, scale_b=None, partial_dtype="f32"):
    """The same result restricted to the global rows `rows` of the local product.

    Returns (own_rows, out_rows): own_rows is len(rows) x N float64; out_rows has
    the reduced value for rows that fall in this rank's shard R_rank and NaN
    rows elsewhere.
    """
    rows = np.asarray(rows, dtype=np.int64)
    own_rows = local_product(a_local_bits, b_local_bits, dtype, scale_a, scale_b, rows=rows)
    M = np.asarray(a_local_bits).shape[0]
    mp = M // P
    out_rows = np.full_like(own_rows, np.nan)
    for t, i in enumerate(rows):
        if i // mp != rank:
            continue
        acc = np.zeros(own_rows.shape[1], dtype=np.float64)
        for p in range(P):
            if p == rank:
                acc += own_rows[t] if partial_dtype == "f32" else codec.bf16_round(own_rows[t])
            elif partial_dtype == "f32":
                acc += np.asarray(partials[p][i - rank * mp], dtype=np.float64)
            else:
                acc += codec.bf16_decode(np.asarray(partials[p][i - rank * mp], dtype=np.uint16))
        out_rows[t] = acc
    return own_rows, out_rows


def gemm_ar(P, rank, a_local_bits, b_local_bits, dtype, partials, peer_rows,
            scale_a=None, scale_b=None, partial_dtype="f32"):
    """One rank's GEMM + all-reduce.

    partials:  as for gemm_rs.
    peer_rows: [P][M/P][N] bf16 bit patterns (uint16); block q != rank is the
               reduced, rounded row block R_q that rank q hands out.  Block
               `rank` is ignored.
    Returns a dict:
      own, outgoing   as gemm_rs;
      out             M/P x N float64, this rank's reduced rows, not rounded;
      bcast_bf16      M/P x N uint16: `out` rounded once, what every rank receives;
      full_bf16       M x N uint16: this rank's copy of the result (own rows
                      rounded, the others as received).
    """
    rs = gemm_rs(P, rank, a_local_bits, b_local_bits, dtype, partials, scale_a, scale_b, partial_dtype)
    mp, N = rs["out"].shape
    peer_rows = np.asarray(peer_rows)
    if peer_rows.shape != (P, mp, N) or peer_rows.dtype != np.uint16:
        raise ValueError(f"peer_rows must be uint16 of shape {(P, mp, N)}")
    full = np.empty((P, mp, N), dtype=np.uint16)
    for q in range(P):
        full[q] = rs["out_bf16"] if q == rank else peer_rows[q]
    return {"own": rs["own"], "outgoing": rs["outgoing"], "out": rs["out"],
            "bcast_bf16": rs["out_bf16"], "full_bf16": full.reshape(P * mp, N)}


def reduce_partials(partials):
    """Sum of the P float32 partial slots, slot order 0..P-1, in float64: [M/P][N]."""
    partials = np.asarray(partials)
    out = np.zeros(partials.shape[1:], dtype=np.float64)
    for p in range(partials.shape[0]):
        out += partials[p].astype(np.float64)
    return out


def gather_chunks(chunks):
    """A_gathered = the P row-chunks stacked in rank order (chunk q = rows R_q)."""
    return np.concatenate([np.asarray(c) for c in chunks], axis=0)


ACTIVATIONS = ("none", "relu", "gelu_tanh", "silu")


def activation(x, kind):
    """The non-linearity between the two GEMMs of the tensor-parallel MLP (section 4.1 asks for one without
    fixing which; these are the usual choices), elementwise in float64:
      relu(x) = max(x, 0);  silu(x) = x / (1 + exp(-x));
      gelu_tanh(x) = x/2 * (1 + tanh( sqrt(2/pi) * (x + 0.044715 x^3) )).
    """
    x = np.asarray(x, dtype=np.float64)
    if kind in (None, "none"):
        return x
    if kind == "relu":
        return np.maximum(x, 0.0)
    if kind == "silu":
        return x / (1.0 + np.exp(-x))
    if kind == "gelu_tanh":
        return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))
    raise ValueError(f"unknown activation {kind!r}")


def gather_kchunks(chunks):
    """A gathered along its LAST dimension (appendix "Additional collective performance": all-gather along the
    tensor dimension): chunk q = columns K_q = [q*K/P, (q+1)*K/P) of every row.  The GEMM that follows is ag_gemm."""
    return np.concatenate([np.asarray(c) for c in chunks], axis=1)


def ag_gemm(P, rank, a_gathered_bits, b_local_bits, dtype,
            scale_a=None, scale_b=None, rows=None, act="none"):
    """One rank's all-gather + GEMM: C[:, N_rank] = act( A . B[:, N_rank] ).

    a_gathered_bits: M x K (all P chunks in place), b_local_bits: K x N/P.
    Returns a dict: C (M x N/P float64, or len(rows) x N/P), C_bf16 (uint16).
    """
    M = np.asarray(a_gathered_bits).shape[0]
    if M % P:
        raise ValueError("M must be a multiple of P")
    if not 0 <= rank < P:
        raise ValueError("rank out of range")
    c = activation(local_product(a_gathered_bits, b_local_bits, dtype, scale_a, scale_b, rows=rows), act)
    return {"C": c, "C_bf16": codec.bf16_encode(c)}


def mlp_block(P, rank, x_gathered_bits, w1_local_bits, w2_local_bits, partials, act="silu"):
    """The tensor-parallel MLP of section 4.1 on rank `rank`, bf16 throughout:
        H = bf16( act( X . W1[:, I_rank] ) )          all-gather + GEMM, column-sharded weights (M x I/P)
        out = sum_p partial_p,  own partial = H . W2[I_rank, :]    GEMM + reduce-scatter, row-sharded weights
    H is rounded to bf16 between the two GEMMs because it is stored as the second GEMM's operand.
    Returns a dict: H_bf16 (uint16), and the gemm_rs result on it (own, outgoing, out, out_bf16).
    """
    h = ag_gemm(P, rank, x_gathered_bits, w1_local_bits, "bf16", act=act)
    res = gemm_rs(P, rank, h["C_bf16"], w2_local_bits, "bf16", partials)
    res["H_bf16"] = h["C_bf16"]
    return res


def abs_product(a_bits, b_bits, dtype, scale_a=None, scale_b=None, rows=None):
    """|scale| * |A| . |B|: the magnitude sum that bounds float32 accumulation error."""
    a_bits = np.asarray(a_bits)
    if rows is not None:
        a_bits = a_bits[np.asarray(rows, dtype=np.int64)]
    a = np.abs(codec.decode(a_bits, dtype))
    b = np.abs(codec.decode(np.asarray(b_bits), dtype))
    return abs(_scale(scale_a, scale_b)) * (a @ b)
