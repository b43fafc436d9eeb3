"""ctypes binding of libpk.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/pk.h.  Tensors are torch CUDA tensors (PyTorch is used for device
memory and streams only); their data pointers are passed through unchanged.
There is no fallback: if libpk.so has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpk.so")

OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_ALIGN, ERR_RANK, ERR_ARG, ERR_HIP, ERR_TIMEOUT = range(9)
BF16, FP8_E4M3 = 0, 1
PHASE_GEMM, PHASE_REDUCE, PHASE_ALL, PHASE_WAIT, PHASE_OVERLAP = 1, 2, 3, 4, 8
AR_ROWS = 8
ACTIVATIONS = {"none": 0, "relu": 1, "gelu_tanh": 2, "silu": 3}
PARTIAL_F32, PARTIAL_BF16 = 0, 1
PARTIALS = {"f32": PARTIAL_F32, "bf16": PARTIAL_BF16}
EMU_MAX_ORDER = 64
DTYPES = {"bf16": BF16, "fp8": FP8_E4M3}
B_LAYOUTS = {"kn": 0, "nk": 1, 0: 0, 1: 1}          # "kn": K x N row-major (default); "nk": N x K row-major (k-contiguous)

EXPORTS = ["pk_version", "pk_status_str", "pk_gemm_rs_plan", "pk_gemm_rs", "pk_ag_gemm_plan", "pk_ag_gemm",
           "pk_emu_deliver_chunks", "pk_emu_deliver_partials", "pk_probe_mfma", "pk_partition_create", "pk_partition_destroy",
           "pk_gemm_ar_plan", "pk_gemm_ar", "pk_emu_deliver_chunks_dma",
           "pk_gemm_rs_cols_plan", "pk_gemm_rs_cols", "pk_ag_gemm_k_plan", "pk_ag_gemm_k",
           "pk_emu_deliver_kchunks_dma", "pk_ag_gemm_static"]


class Plan(ctypes.Structure):
    _fields_ = [("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("tiles_m", ctypes.c_int32), ("tiles_n", ctypes.c_int32),
                ("flags_per_slot", ctypes.c_int64),
                ("local_m", ctypes.c_int64), ("local_n", ctypes.c_int64), ("local_k", ctypes.c_int64),
                ("ar_flags_per_slot", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64)]


class PkError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_str(code)} (pk_status {code})")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_13940_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, u32, u64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p
        L.pk_version.restype = ctypes.c_int
        L.pk_status_str.restype = ctypes.c_char_p
        L.pk_status_str.argtypes = [i32]
        for f in (L.pk_gemm_rs_plan, L.pk_ag_gemm_plan, L.pk_gemm_ar_plan, L.pk_gemm_rs_cols_plan, L.pk_ag_gemm_k_plan):
            f.restype = i32
            f.argtypes = [i32, i64, i64, i64, i32, ctypes.POINTER(Plan)]
        L.pk_gemm_rs.restype = i32
        rs_args = [i32, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, u32, vp, u32, i32, i32, vp, u64, vp]
        ag_args = [i32, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp, u32, vp, i32, i32, vp, u64, vp]
        L.pk_gemm_rs.argtypes = rs_args[:19] + [i32, vp, ctypes.c_size_t] + rs_args[19:]
        L.pk_ag_gemm.restype = i32
        L.pk_ag_gemm.argtypes = ag_args[:15] + [i32, vp, ctypes.c_size_t] + ag_args[15:]
        L.pk_emu_deliver_chunks.restype = i32
        L.pk_emu_deliver_chunks.argtypes = [i32, i64, i64, i32, vp, vp, vp, u32, ctypes.POINTER(i32), i32, u32, i32, vp, vp]
        L.pk_emu_deliver_partials.restype = i32
        L.pk_emu_deliver_partials.argtypes = [i32, i64, i64, i32, i32, vp, vp, vp, u32, ctypes.POINTER(i32), i32, u32, i32, vp]
        L.pk_probe_mfma.restype = i32
        L.pk_probe_mfma.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pk_gemm_rs_cols.restype = i32
        L.pk_gemm_rs_cols.argtypes = rs_args
        L.pk_gemm_ar.restype = i32
        L.pk_gemm_ar.argtypes = [i32, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, i32,
                                 i32, vp, u64, vp]
        L.pk_ag_gemm_k.restype = i32
        L.pk_ag_gemm_k.argtypes = ag_args
        L.pk_ag_gemm_static.restype = i32
        L.pk_ag_gemm_static.argtypes = ag_args
        L.pk_emu_deliver_kchunks_dma.restype = i32
        L.pk_emu_deliver_kchunks_dma.argtypes = [i32, i64, i64, i32, vp, vp, vp, u32, ctypes.POINTER(i32), i32, vp]
        L.pk_emu_deliver_chunks_dma.restype = i32
        L.pk_emu_deliver_chunks_dma.argtypes = [i32, i64, i64, i32, vp, vp, vp, u32, ctypes.POINTER(i32), i32, vp]
        L.pk_partition_create.restype = i32
        L.pk_partition_create.argtypes = [i32, ctypes.POINTER(vp), ctypes.POINTER(vp)]
        L.pk_partition_destroy.restype = i32
        L.pk_partition_destroy.argtypes = [vp, vp]
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libpk takes contiguous device tensors")
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dt(dtype):
    return DTYPES[dtype] if isinstance(dtype, str) else int(dtype)


def _pdt(partial_dtype):
    return PARTIALS[partial_dtype] if isinstance(partial_dtype, str) else int(partial_dtype)


def _check(code, where):
    if code != OK:
        raise PkError(code, where)


def pk_version():
    return lib().pk_version()


def status_str(code):
    return lib().pk_status_str(int(code)).decode()


def pk_gemm_rs_plan(P, M, N, K, dtype):
    p = Plan()
    _check(lib().pk_gemm_rs_plan(P, M, N, K, _dt(dtype), ctypes.byref(p)), "pk_gemm_rs_plan")
    return p


def pk_ag_gemm_plan(P, M, N, K, dtype):
    p = Plan()
    _check(lib().pk_ag_gemm_plan(P, M, N, K, _dt(dtype), ctypes.byref(p)), "pk_ag_gemm_plan")
    return p


def pk_gemm_rs(P, rank, M, N, K, dtype, A_local, B_local, scale_a, scale_b, partials, outgoing,
               flags_in, flags_out, epoch, out_shard, phases, status, timeout_us=0, stream=None, comm_cus=0,
               partial_dtype="f32", workspace=None, b_layout="kn"):
    _check(lib().pk_gemm_rs(P, rank, M, N, K, _dt(dtype), _ptr(A_local), _ptr(B_local), _ptr(scale_a), _ptr(scale_b),
                            _ptr(partials), _ptr(outgoing), _ptr(flags_in), _ptr(flags_out), epoch,
                            _ptr(out_shard), phases, comm_cus, _pdt(partial_dtype), B_LAYOUTS[b_layout], _ptr(workspace),
                            _nbytes(workspace),
                            _ptr(status), timeout_us, _stream(stream)), "pk_gemm_rs")


def pk_gemm_rs_cols_plan(P, M, N, K, dtype):
    p = Plan()
    _check(lib().pk_gemm_rs_cols_plan(P, M, N, K, _dt(dtype), ctypes.byref(p)), "pk_gemm_rs_cols_plan")
    return p


def pk_gemm_rs_cols(P, rank, M, N, K, dtype, A_local, B_local, scale_a, scale_b, partials, outgoing,
                    flags_in, flags_out, epoch, out_shard, phases, status, timeout_us=0, stream=None, comm_cus=0,
                    partial_dtype="f32"):
    _check(lib().pk_gemm_rs_cols(P, rank, M, N, K, _dt(dtype), _ptr(A_local), _ptr(B_local), _ptr(scale_a),
                                 _ptr(scale_b), _ptr(partials), _ptr(outgoing), _ptr(flags_in), _ptr(flags_out), epoch,
                                 _ptr(out_shard), phases, comm_cus, _pdt(partial_dtype), _ptr(status), timeout_us,
                                 _stream(stream)), "pk_gemm_rs_cols")


def pk_gemm_ar_plan(P, M, N, K, dtype):
    p = Plan()
    _check(lib().pk_gemm_ar_plan(P, M, N, K, _dt(dtype), ctypes.byref(p)), "pk_gemm_ar_plan")
    return p


def pk_gemm_ar(P, rank, M, N, K, dtype, A_local, B_local, scale_a, scale_b, partials, outgoing, flags_in, flags_out,
               out_full, bcast_out, ar_flags_in, ar_flags_out, epoch, phases, status, timeout_us=0, stream=None,
               comm_cus=0, partial_dtype="f32"):
    _check(lib().pk_gemm_ar(P, rank, M, N, K, _dt(dtype), _ptr(A_local), _ptr(B_local), _ptr(scale_a), _ptr(scale_b),
                            _ptr(partials), _ptr(outgoing), _ptr(flags_in), _ptr(flags_out), _ptr(out_full),
                            _ptr(bcast_out), _ptr(ar_flags_in), _ptr(ar_flags_out), epoch, phases, comm_cus,
                            _pdt(partial_dtype), _ptr(status), timeout_us, _stream(stream)), "pk_gemm_ar")


def pk_ag_gemm(P, rank, M, N, K, dtype, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch,
               C_local, status, timeout_us=0, stream=None, comm_cus=0, act="none", workspace=None, b_layout="kn"):
    _check(lib().pk_ag_gemm(P, rank, M, N, K, _dt(dtype), _ptr(A_gathered), _ptr(B_local), _ptr(scale_a),
                            _ptr(scale_b), _ptr(chunk_flags), epoch, _ptr(C_local), comm_cus,
                            ACTIVATIONS[act] if isinstance(act, str) else int(act), B_LAYOUTS[b_layout], _ptr(workspace),
                            _nbytes(workspace),
                            _ptr(status), timeout_us, _stream(stream)), "pk_ag_gemm")


def pk_ag_gemm_static(P, rank, M, N, K, dtype, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch,
                      C_local, status, timeout_us=0, stream=None, comm_cus=0, act="none"):
    _check(lib().pk_ag_gemm_static(P, rank, M, N, K, _dt(dtype), _ptr(A_gathered), _ptr(B_local), _ptr(scale_a),
                                   _ptr(scale_b), _ptr(chunk_flags), epoch, _ptr(C_local), comm_cus,
                                   ACTIVATIONS[act] if isinstance(act, str) else int(act), _ptr(status),
                                   timeout_us, _stream(stream)), "pk_ag_gemm_static")


def pk_ag_gemm_k_plan(P, M, N, K, dtype):
    p = Plan()
    _check(lib().pk_ag_gemm_k_plan(P, M, N, K, _dt(dtype), ctypes.byref(p)), "pk_ag_gemm_k_plan")
    return p


def pk_ag_gemm_k(P, rank, M, N, K, dtype, A_gathered, B_local, scale_a, scale_b, chunk_flags, epoch,
                 C_local, status, timeout_us=0, stream=None, comm_cus=0, act="none"):
    _check(lib().pk_ag_gemm_k(P, rank, M, N, K, _dt(dtype), _ptr(A_gathered), _ptr(B_local), _ptr(scale_a),
                              _ptr(scale_b), _ptr(chunk_flags), epoch, _ptr(C_local), comm_cus,
                              ACTIVATIONS[act] if isinstance(act, str) else int(act), _ptr(status),
                              timeout_us, _stream(stream)), "pk_ag_gemm_k")


def _order(order):
    arr = (ctypes.c_int * max(1, len(order)))(*order)
    return arr, len(order)


def pk_emu_deliver_chunks(P, M, K, elem_bytes, staging, A_gathered, chunk_flags, epoch, order, gap_us,
                          counters, stream=None, n_wg=0):
    arr, n = _order(order)
    _check(lib().pk_emu_deliver_chunks(P, M, K, elem_bytes, _ptr(staging), _ptr(A_gathered), _ptr(chunk_flags),
                                       epoch, arr, n, gap_us, n_wg, _ptr(counters), _stream(stream)),
           "pk_emu_deliver_chunks")


def pk_emu_deliver_chunks_dma(P, M, K, elem_bytes, staging, A_gathered, chunk_flags, epoch, order, stream=None):
    arr, n = _order(order)
    _check(lib().pk_emu_deliver_chunks_dma(P, M, K, elem_bytes, _ptr(staging), _ptr(A_gathered), _ptr(chunk_flags), epoch,
                                           arr, n, _stream(stream)), "pk_emu_deliver_chunks_dma")


def pk_emu_deliver_kchunks_dma(P, M, K, elem_bytes, staging, A_gathered, chunk_flags, epoch, order, stream=None):
    arr, n = _order(order)
    _check(lib().pk_emu_deliver_kchunks_dma(P, M, K, elem_bytes, _ptr(staging), _ptr(A_gathered), _ptr(chunk_flags), epoch,
                                            arr, n, _stream(stream)), "pk_emu_deliver_kchunks_dma")


def pk_emu_deliver_partials(P, M, N, tile_m, tile_n, staging, partials, flags_in, epoch, order, gap_us,
                            stream=None, n_wg=0):
    arr, n = _order(order)
    _check(lib().pk_emu_deliver_partials(P, M, N, tile_m, tile_n, _ptr(staging), _ptr(partials), _ptr(flags_in),
                                         epoch, arr, n, gap_us, n_wg, _stream(stream)), "pk_emu_deliver_partials")


def pk_probe_mfma(iters, random_operands, report, stream=None):
    """Launches the register-only MFMA loop; returns the flop count of the launch (time it with events)."""
    flops = ctypes.c_double(0.0)
    _check(lib().pk_probe_mfma(iters, 1 if random_operands else 0, _ptr(report), ctypes.byref(flops), _stream(stream)),
           "pk_probe_mfma")
    return flops.value


def pk_partition_create(comm_cus):
    """Two hipStream_t handles (ints) on disjoint compute units: (compute_stream, comm_stream)."""
    a, b = ctypes.c_void_p(), ctypes.c_void_p()
    _check(lib().pk_partition_create(comm_cus, ctypes.byref(a), ctypes.byref(b)), "pk_partition_create")
    return a.value, b.value


def pk_partition_destroy(compute_stream, comm_stream):
    _check(lib().pk_partition_destroy(compute_stream, comm_stream), "pk_partition_destroy")
