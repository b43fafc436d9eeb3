"""pk_ag_gemm_static (the entry point that allocates nothing: stream-K workspace in the library's own scratch array)
against pk_ag_gemm with a caller workspace, through the C ABI: two calls in a row, the second on a smaller problem.
Both run the same kernels on the same piece order, so the outputs must be bit-identical."""
import numpy as np
import pytest
import torch

from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu


def both(P, rank, M, N, K, dtype, seed, epoch):
    inp = wl.ag_gemm_inputs(P, M, N, K, dtype, rank, seed=seed)
    ref = hz.run_ag_gemm(P, rank, M, N, K, dtype, inp["chunks"], inp["B_local"], scale_a=inp["scale_a"],
                         scale_b=inp["scale_b"], workspace=True, epoch=epoch, fetch_A=False)
    assert ref["status"][0] == 0
    npdt = np.uint16 if dtype == "bf16" else np.uint8
    A = hz.elem_view(np.concatenate([np.asarray(c, dtype=npdt) for c in inp["chunks"]], axis=0), dtype)
    B = hz.elem_view(inp["B_local"], dtype)
    sa, sb = hz.scale_t(inp["scale_a"]), hz.scale_t(inp["scale_b"])
    C = torch.full((M, N // P), -1, dtype=torch.int16, device="cuda")
    flags = torch.full((P,), epoch, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    pk.pk_ag_gemm_static(P, rank, M, N, K, dtype, A, B, sa, sb, flags if P > 1 else None, epoch, C, status)
    torch.cuda.synchronize()
    assert status[0].item() == 0, status.tolist()
    assert np.array_equal(hz.bits_of(C), ref["C_bits"])


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    # 288 tiles of 256 x 256: one whole round on 256 compute units and a stream-K tail of 32 tiles
    both(2, 1, 4608, 8192, 1024, "bf16", seed=41, epoch=9)
    # smaller, and with the small tiles: 288 tiles of 128 x 128; the scratch still holds the first call's flags and pieces
    both(1, 0, 2304, 2048, 1024, "bf16", seed=42, epoch=3)
    # fp8, an epoch below the previous ones
    both(2, 0, 4608, 8192, 2048, "fp8", seed=43, epoch=1)
