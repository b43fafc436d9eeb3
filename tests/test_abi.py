"""The C-ABI boundary without a GPU: the library loads, exports what include/pk.h declares, and its host-side
validation returns the documented codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2511_13940_amd import pk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "pk.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pk_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = pk.lib()
    names = _declared()
    assert set(names) == set(pk.EXPORTS), names
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    assert pk.pk_version() >= 1
    seen = {pk.status_str(c) for c in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert pk.status_str(99) == "unknown status"


def test_plans():
    p = pk.pk_gemm_rs_plan(8, 8192, 8192, 28672, "bf16")
    assert (p.tile_m, p.tile_n, p.tiles_m, p.tiles_n, p.flags_per_slot) == (256, 256, 4, 32, 128)
    assert (p.local_m, p.local_n, p.local_k) == (8192, 8192, 3584)
    p = pk.pk_ag_gemm_plan(8, 8192, 28672, 8192, "bf16")
    assert (p.tile_m, p.tiles_m, p.tiles_n, p.local_n, p.local_k) == (256, 4, 14, 3584, 8192)
    p = pk.pk_gemm_rs_plan(2, 256, 256, 512, "bf16")
    assert (p.tile_m, p.tile_n, p.tiles_m, p.tiles_n) == (128, 128, 1, 2)
    p = pk.pk_gemm_rs_plan(2, 2 * 200, 264, 256, "bf16")            # ragged: edge tiles are partial
    assert (p.tiles_m, p.tiles_n) == (2, 3)
    p = pk.pk_gemm_rs_plan(8, 16384, 16384, 16384, "fp8")
    assert (p.tile_m, p.flags_per_slot, p.local_k) == (256, 8 * 64, 2048)


@pytest.mark.parametrize("args,code", [
    ((0, 256, 256, 512, pk.BF16), pk.ERR_SHAPE),          # P < 1
    ((3, 256, 256, 512, pk.BF16), pk.ERR_SHAPE),          # M % P
    ((2, 256, 256, 510, pk.BF16), pk.ERR_SHAPE),          # K/P not a multiple of 64
    ((2, 256, 252, 512, pk.BF16), pk.ERR_SHAPE),          # N % 8
    ((2, 256, 256, 384, pk.FP8_E4M3), pk.ERR_SHAPE),      # fp8: K/P % 128
    ((2, 256, 256, 512, 7), pk.ERR_DTYPE),
    ((2, 0, 256, 512, pk.BF16), pk.ERR_SHAPE),            # empty problem
])
def test_plan_errors(args, code):
    plan = pk.Plan()
    assert pk.lib().pk_gemm_rs_plan(*args, ctypes.byref(plan)) == code
    assert pk.lib().pk_gemm_rs_plan(2, 256, 256, 512, pk.BF16, None) == pk.ERR_NULL


def _rs(P=2, rank=0, M=256, N=256, K=512, dt=pk.BF16, A=0x1000, B=0x2000, sa=None, sb=None, part=0x3000,
        outg=0x4000, fin=0x5000, fout=0x6000, out=0x7000, phases=3, status=0x8000, pdt=0, ws=None, ws_bytes=0, bl=0):
    return pk.lib().pk_gemm_rs(P, rank, M, N, K, dt, A, B, sa, sb, part, outg, fin, fout, 1, out, phases, 0, pdt, bl, ws, ws_bytes,
                               status, 0, None)


def test_gemm_rs_argument_errors_launch_nothing():
    """Fake non-null pointers: every call below must be rejected on the host (a launch would need a GPU)."""
    assert _rs(rank=2) == pk.ERR_RANK
    assert _rs(rank=-1) == pk.ERR_RANK
    assert _rs(A=None) == pk.ERR_NULL
    assert _rs(part=None) == pk.ERR_NULL
    assert _rs(outg=None) == pk.ERR_NULL
    assert _rs(status=None) == pk.ERR_NULL
    assert _rs(out=None) == pk.ERR_NULL
    assert _rs(A=0x1008) == pk.ERR_ALIGN
    assert _rs(out=0x7004) == pk.ERR_ALIGN
    assert _rs(phases=0) == pk.ERR_ARG
    assert _rs(phases=4) == pk.ERR_ARG
    assert _rs(dt=pk.FP8_E4M3, K=256) == pk.ERR_DTYPE       # fp8 without scales
    assert _rs(M=255) == pk.ERR_SHAPE
    assert _rs(dt=5) == pk.ERR_DTYPE
    assert pk.lib().pk_gemm_rs(2, 0, 256, 256, 512, pk.BF16, 0x1000, 0x2000, None, None, 0x3000, 0x4000, 0x5000, 0x6000, 1,
                               0x7000, 3, -8, 0, 0, None, 0, 0x8000, 0, None) == pk.ERR_ARG      # comm_cus
    assert _rs(bl=2) == pk.ERR_ARG
    assert _rs(bl=1, pdt=1) == pk.ERR_ARG                    # k-contiguous B is built for fp32 slots only
    assert _rs(ws=0x9004, ws_bytes=1 << 30) == pk.ERR_ALIGN
    assert _rs(pdt=2) == pk.ERR_DTYPE
    assert _rs(pdt=-1) == pk.ERR_DTYPE


def test_ag_gemm_argument_errors_launch_nothing():
    f = pk.lib().pk_ag_gemm

    def ag(P=4, rank=0, M=2048, N=4096, K=2048, dt=pk.BF16, A=0x1000, B=0x2000, flags=0x3000, C=0x4000, status=0x5000,
           comm=0, act=0, ws=None, ws_bytes=0, bl=0):
        return f(P, rank, M, N, K, dt, A, B, None, None, flags, 1, C, comm, act, bl, ws, ws_bytes, status, 0, None)

    assert ag(rank=4) == pk.ERR_RANK
    assert ag(N=4098) == pk.ERR_SHAPE        # N % P
    assert ag(N=4 * 1028) == pk.ERR_SHAPE    # (N/P) % 8
    assert ag(K=2000) == pk.ERR_SHAPE
    assert ag(A=None) == pk.ERR_NULL
    assert ag(flags=None) == pk.ERR_NULL
    assert ag(C=0x4002) == pk.ERR_ALIGN
    assert ag(dt=pk.FP8_E4M3) == pk.ERR_DTYPE
    assert ag(comm=-1) == pk.ERR_ARG
    assert ag(act=4) == pk.ERR_ARG
    assert ag(act=-1) == pk.ERR_ARG
    assert ag(ws=0x9008, ws_bytes=1 << 30) == pk.ERR_ALIGN
    assert ag(bl=-1) == pk.ERR_ARG


def test_emulator_argument_errors_launch_nothing():
    L = pk.lib()
    order = (ctypes.c_int * 3)(1, 2, 2)
    assert L.pk_emu_deliver_chunks(4, 2048, 2048, 2, 0x1000, 0x2000, 0x3000, 1, order, 3, 0, 0, 0x4000, None) == pk.ERR_ARG
    order = (ctypes.c_int * 3)(1, 2, 4)
    assert L.pk_emu_deliver_chunks(4, 2048, 2048, 2, 0x1000, 0x2000, 0x3000, 1, order, 3, 0, 0, 0x4000, None) == pk.ERR_ARG
    order = (ctypes.c_int * 3)(1, 2, 3)
    assert L.pk_emu_deliver_chunks(4, 2048, 2048, 4, 0x1000, 0x2000, 0x3000, 1, order, 3, 0, 0, 0x4000, None) == pk.ERR_DTYPE
    assert L.pk_emu_deliver_chunks(4, 2048, 2048, 2, None, 0x2000, 0x3000, 1, order, 3, 0, 0, 0x4000, None) == pk.ERR_NULL
    assert L.pk_emu_deliver_chunks(4, 2048, 2048, 2, 0x1000, 0x2000, 0x3000, 1, order, 0, 0, 0, 0x4000, None) == pk.OK
    assert L.pk_emu_deliver_chunks_dma(4, 2048, 2048, 2, None, 0x2000, 0x3000, 1, order, 3, None) == pk.ERR_NULL
    assert L.pk_emu_deliver_chunks_dma(4, 2047, 2048, 2, 0x1000, 0x2000, 0x3000, 1, order, 3, None) == pk.ERR_SHAPE
    assert L.pk_emu_deliver_chunks_dma(4, 2048, 2048, 2, 0x1000, 0x2000, 0x3000, 1, order, 0, None) == pk.OK
    assert L.pk_emu_deliver_partials(4, 2048, 2048, 128, 128, 0x1000, 0x2000, 0x3000, 1, order, 65, 0, 0, None) == pk.ERR_ARG
    assert L.pk_emu_deliver_partials(4, 2048, 2048, 128, 130, 0x1000, 0x2000, 0x3000, 1, order, 3, 0, 0, None) == pk.ERR_ARG
    assert L.pk_emu_deliver_partials(4, 2048, 2048, 128, 128, 0x1000, 0x2000, 0x3000, 1, order, 0, 0, 0, None) == pk.OK


def test_gemm_ar_plan_and_argument_errors_launch_nothing():
    p = pk.pk_gemm_ar_plan(8, 8192, 8192, 28672, "bf16")
    assert (p.tile_m, p.tile_n, p.flags_per_slot) == (256, 256, 4 * 32)
    assert p.ar_flags_per_slot == (1024 // pk.AR_ROWS) * 32
    assert pk.pk_gemm_rs_plan(8, 8192, 8192, 28672, "bf16").ar_flags_per_slot == 0
    p = pk.pk_gemm_ar_plan(2, 2 * 100, 264, 256, "bf16")                  # ragged: 100 rows -> 13 row blocks
    assert p.ar_flags_per_slot == 13 * p.tiles_n
    f = pk.lib().pk_gemm_ar

    def ar(P=2, rank=0, M=256, N=256, K=512, full=0x9000, bc=0xA000, ai=0xB000, ao=0xC000, phases=7, status=0x8000,
           part=0x3000, pdt=0):
        return f(P, rank, M, N, K, pk.BF16, 0x1000, 0x2000, None, None, part, 0x4000, 0x5000, 0x6000, full, bc, ai, ao,
                 1, phases, 0, pdt, status, 0, None)

    assert ar(phases=0) == pk.ERR_ARG
    assert ar(phases=8) == pk.ERR_ARG
    assert ar(full=None) == pk.ERR_NULL
    assert ar(bc=None) == pk.ERR_NULL
    assert ar(ai=None) == pk.ERR_NULL
    assert ar(ao=None) == pk.ERR_NULL
    assert ar(status=None) == pk.ERR_NULL
    assert ar(full=0x9008) == pk.ERR_ALIGN
    assert ar(rank=2) == pk.ERR_RANK
    assert ar(M=255) == pk.ERR_SHAPE
    assert ar(part=None) == pk.ERR_NULL
    assert ar(pdt=3) == pk.ERR_DTYPE


def test_partition_and_probe_argument_errors_launch_nothing():
    L = pk.lib()
    a, b = ctypes.c_void_p(), ctypes.c_void_p()
    assert L.pk_partition_create(32, None, ctypes.byref(b)) == pk.ERR_NULL
    assert L.pk_partition_create(32, ctypes.byref(a), None) == pk.ERR_NULL
    for bad in (0, 4, 12, -8, 1 << 20):
        assert L.pk_partition_create(bad, ctypes.byref(a), ctypes.byref(b)) == pk.ERR_ARG
    assert a.value is None and b.value is None
    assert L.pk_partition_destroy(None, None) == pk.OK
    assert L.pk_probe_mfma(100, 1, None, None, None) == pk.ERR_NULL
    assert L.pk_probe_mfma(0, 1, 0x1000, None, None) == pk.ERR_ARG


def test_size_limits():
    """32-bit byte offsets inside one operand and inside one partial slot; the slots together may exceed 4 GiB."""
    p = pk.pk_gemm_rs_plan(8, 32768, 32768, 8 * 8192, "bf16")                  # the paper's Table 3 size: 8 slots of 512 MiB
    assert (p.tiles_m, p.tiles_n, p.local_k) == (16, 128, 8192)
    plan = pk.Plan()
    L = pk.lib()
    assert L.pk_gemm_rs_plan(2, 65536, 32768, 2 * 64, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE     # one slot = 4 GiB
    assert L.pk_gemm_rs_plan(8, 32768, 32768, 8 * 65536, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE  # A_local = 4 GiB
    assert L.pk_ag_gemm_plan(8, 32768, 8 * 8192, 65536, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE   # A_gathered = 4 GiB


def test_binding_raises_pk_error():
    with pytest.raises(pk.PkError) as e:
        pk.pk_gemm_rs_plan(3, 256, 256, 512, "bf16")
    assert e.value.code == pk.ERR_SHAPE


def test_gemm_rs_cols_plan_and_argument_errors_launch_nothing():
    p = pk.pk_gemm_rs_cols_plan(8, 8192, 8192, 28672, "bf16")
    assert (p.tile_m, p.tile_n, p.tiles_m, p.tiles_n, p.flags_per_slot) == (256, 256, 32, 4, 128)
    assert (p.local_m, p.local_n, p.local_k) == (8192, 8192, 3584)
    p = pk.pk_gemm_rs_cols_plan(4, 136, 4 * 264, 1024, "bf16")             # M not a multiple of P is fine here
    assert (p.tile_m, p.tiles_m, p.tiles_n) == (128, 2, 3)
    plan = pk.Plan()
    L = pk.lib()
    assert L.pk_gemm_rs_cols_plan(4, 136, 4 * 260, 1024, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE     # (N/P) % 8
    assert L.pk_gemm_rs_cols_plan(4, 136, 1058, 1024, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE         # N % P
    assert L.pk_gemm_rs_cols_plan(4, 136, 1056, 1000, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE         # K/P % 64
    assert L.pk_gemm_rs_cols_plan(4, 136, 1056, 1024, pk.BF16, None) == pk.ERR_NULL

    def rs(rank=0, part=0x3000, phases=3, pdt=0, out=0x7000):
        return L.pk_gemm_rs_cols(2, rank, 300, 512, 512, pk.BF16, 0x1000, 0x2000, None, None, part, 0x4000, 0x5000, 0x6000, 1,
                                 out, phases, 0, pdt, 0x8000, 0, None)
    assert rs(rank=2) == pk.ERR_RANK
    assert rs(part=None) == pk.ERR_NULL
    assert rs(phases=0) == pk.ERR_ARG
    assert rs(pdt=7) == pk.ERR_DTYPE
    assert rs(out=0x7001) == pk.ERR_ALIGN


def test_ag_gemm_k_plan_and_argument_errors_launch_nothing():
    p = pk.pk_ag_gemm_k_plan(8, 8192, 28672, 8192, "bf16")
    assert (p.tile_m, p.tile_n, p.tiles_m, p.tiles_n) == (256, 256, 32, 14)
    assert (p.local_m, p.local_n, p.local_k) == (8192, 3584, 8192)
    p = pk.pk_ag_gemm_k_plan(4, 200, 4 * 264, 4 * 128, "bf16")              # M need not divide by P
    assert (p.tile_m, p.tiles_m, p.tiles_n) == (128, 2, 3)
    L = pk.lib()
    plan = pk.Plan()
    assert L.pk_ag_gemm_k_plan(4, 200, 1056, 4 * 96, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE          # (K/P) % 64
    assert L.pk_ag_gemm_k_plan(4, 200, 1056, 510, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE             # K % P
    assert L.pk_ag_gemm_k_plan(4, 200, 1058, 512, pk.BF16, ctypes.byref(plan)) == pk.ERR_SHAPE             # N % P

    def ag(rank=0, A=0x1000, flags=0x3000, act=0):
        return L.pk_ag_gemm_k(4, rank, 200, 1056, 512, pk.BF16, A, 0x2000, None, None, flags, 1, 0x4000, 0, act, 0x5000, 0, None)
    assert ag(rank=4) == pk.ERR_RANK
    assert ag(A=None) == pk.ERR_NULL
    assert ag(flags=None) == pk.ERR_NULL
    assert ag(act=9) == pk.ERR_ARG
    order = (ctypes.c_int * 3)(1, 2, 3)
    assert L.pk_emu_deliver_kchunks_dma(4, 200, 510, 2, 0x1000, 0x2000, 0x3000, 1, order, 3, None) == pk.ERR_SHAPE
    assert L.pk_emu_deliver_kchunks_dma(4, 200, 512, 2, None, 0x2000, 0x3000, 1, order, 3, None) == pk.ERR_NULL
    assert L.pk_emu_deliver_kchunks_dma(4, 200, 512, 2, 0x1000, 0x2000, 0x3000, 1, order, 0, None) == pk.OK


def test_header_and_library_work_from_plain_c(tmp_path):
    """include/pk.h compiles as C99 and a C program linked against libpk.so gets the same answers."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    here = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(here)
    libdir = os.path.dirname(pk.LIB_PATH)
    exe = str(tmp_path / "c_abi_check")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-I", os.path.join(root, "include"), os.path.join(here, "c_abi_check.c"),
                    "-L", libdir, "-l:libpk.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib",
                    "-Wl,--allow-shlib-undefined", "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert "c abi ok" in out.stdout
