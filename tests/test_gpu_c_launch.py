"""Both hot-path entry points driven from a plain C translation unit (tests/c_abi_launch.c: include/pk.h and the HIP
runtime's C interface, hipMalloc'd buffers, integer-exact expected bits computed in C)."""
import ctypes
import os

import pytest

pytestmark = pytest.mark.gpu


def test_c_caller_launches_both_entry_points_and_gets_exact_bits():
    here = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(here, "libc_abi_launch.so")
    assert os.path.exists(path), "tests/libc_abi_launch.so is not built: run python -m paper_2511_13940_amd.build"
    lib = ctypes.CDLL(path)
    lib.pk_c_abi_launch.restype = ctypes.c_int
    rc = lib.pk_c_abi_launch()
    assert rc == 0, f"pk_c_abi_launch returned {rc} (1-6: wrong result, 100: HIP error, 101: library error; see stderr)"
