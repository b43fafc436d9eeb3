"""The ops only launch kernels on the caller's stream, so a sequence of them can be captured into a HIP graph once the
kernels have run once eagerly (their LDS-size attribute is set on first use).  Each replay, with eager work and
synchronisation in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2511_13940_amd import pk, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu


def test_captured_mlp_block_replays_bit_identically():
    P, rank, M, D, I = 4, 2, 1024, 512, 2048          # AG+GEMM: X (M x D) . W1[:, I_r] -> H (M x I/P); GEMM+RS: H . W2[I_r, :]
    inp1 = wl.ag_gemm_inputs(P, M, I, D, "bf16", rank, seed=51)
    inp2 = wl.gemm_rs_inputs(P, M, D, I, "bf16", rank, seed=52)
    X = hz.elem_view(np.concatenate(inp1["chunks"], axis=0), "bf16")
    W1, W2 = hz.elem_view(inp1["B_local"], "bf16"), hz.elem_view(inp2["B_local"], "bf16")
    plan = pk.pk_gemm_rs_plan(P, M, D, I, "bf16")
    mp = M // P
    part = hz.dev(inp2["partials"])
    outgoing = torch.zeros((P, mp, D), dtype=torch.float32, device="cuda")
    flags_in = torch.full((P, plan.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    flags_in[rank].zero_()
    flags_out = torch.zeros_like(flags_in)
    chunk_flags = torch.full((P,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    H = torch.zeros((M, I // P), dtype=torch.int16, device="cuda")
    out = torch.zeros((mp, D), dtype=torch.int16, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")

    def block(epoch):
        pk.pk_ag_gemm(P, rank, M, I, D, "bf16", X, W1, None, None, chunk_flags, epoch, H, status, act="silu")
        pk.pk_gemm_rs(P, rank, M, D, I, "bf16", H, W2, None, None, part, outgoing, flags_in, flags_out, epoch, out,
                      pk.PHASE_ALL, status)

    block(1)                                           # eager: also the kernels' one-time set-up
    torch.cuda.synchronize()
    want_out, want_H = out.clone(), H.clone()
    assert status[0].item() == 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        block(2)                                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            block(3)
    torch.cuda.synchronize()
    for i in range(4):
        out.fill_(-1)
        H.fill_(-1)
        outgoing.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum()      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert status[0].item() == 0
        assert torch.equal(H, want_H), f"replay {i}"
        assert torch.equal(out, want_out), f"replay {i}"
        assert torch.isfinite(scratch)
    assert torch.all(flags_in[rank] == 3) and torch.all(flags_out[(rank + 1) % P] == 3)


def test_captured_gemm_rs_with_the_reduce_beside_the_gemm_replays_bit_identically():
    """PK_PHASE_OVERLAP forks to the library's second stream and joins it back: inside a capture that stream becomes part
    of the graph.  The library's stream and events exist from the eager call on."""
    P, rank, M, N, K = 4, 1, 4096, 2048, 1024          # 512 tiles of 128: the own block's rows and the rest, two launches
    inp = wl.gemm_rs_inputs(P, M, N, K, "bf16", rank, seed=53)
    A, B = hz.elem_view(inp["A_local"], "bf16"), hz.elem_view(inp["B_local"], "bf16")
    plan = pk.pk_gemm_rs_plan(P, M, N, K, "bf16")
    mp = M // P
    part = hz.dev(inp["partials"])
    outgoing = torch.zeros((P, mp, N), dtype=torch.float32, device="cuda")
    flags_in = torch.full((P, plan.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    flags_in[rank].zero_()
    flags_out = torch.zeros_like(flags_in)
    out = torch.zeros((mp, N), dtype=torch.int16, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")

    def op(epoch, phases):
        pk.pk_gemm_rs(P, rank, M, N, K, "bf16", A, B, None, None, part, outgoing, flags_in, flags_out, epoch, out, phases,
                      status)

    op(1, pk.PHASE_ALL)
    torch.cuda.synchronize()
    want = out.clone()
    op(2, pk.PHASE_ALL | pk.PHASE_OVERLAP)             # eager: creates the library's second stream
    torch.cuda.synchronize()
    assert status[0].item() == 0 and torch.equal(out, want)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        op(3, pk.PHASE_ALL | pk.PHASE_OVERLAP)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            op(4, pk.PHASE_ALL | pk.PHASE_OVERLAP)
    torch.cuda.synchronize()
    for i in range(4):
        out.fill_(-1)
        part[rank].fill_(float("nan"))
        scratch = torch.randn(1 << 20, device="cuda").sum()      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert status[0].item() == 0
        assert torch.equal(out, want), f"replay {i}"
        assert torch.isfinite(scratch)
    assert torch.all(flags_in[rank] == 4)
