"""Glue for the GPU parity tests: uploads seeded numpy inputs, calls libpk through its binding,
downloads the results.  No arithmetic of the method happens here."""
import numpy as np
import torch

from paper_2511_13940_amd import pk

NAN_POISON = float("nan")


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def elem_view(bits, dtype):
    """numpy uint16/uint8 bit patterns -> device tensor of raw bits."""
    if dtype == "bf16":
        return dev(bits.view(np.int16))
    return dev(bits)


def scale_t(s):
    return None if s is None else torch.tensor([float(s)], dtype=torch.float32, device="cuda")


def bits_of(t):
    """device bf16-bit tensor (int16) -> numpy uint16."""
    return t.cpu().numpy().view(np.uint16)


BF16_NAN = 0x7FC1


def slot_poison(P, mp, N, s16):
    """Partial slots filled with NaN: fp32, or bf16 bit patterns held in an int16 tensor."""
    if s16:
        return dev(np.full((P, mp, N), BF16_NAN, dtype=np.uint16).view(np.int16))
    return torch.full((P, mp, N), NAN_POISON, dtype=torch.float32, device="cuda")


def slot_upload(partials, s16):
    if s16:
        return dev(np.ascontiguousarray(partials, dtype=np.uint16).view(np.int16))
    return dev(partials.astype(np.float32))


def slot_download(t, s16):
    return bits_of(t) if s16 else t.cpu().numpy()


def make_workspace(plan, workspace):
    """None -> no workspace; True -> a zeroed one of the size the plan asks for; a tensor -> that tensor."""
    if workspace is None or workspace is False:
        return None
    if workspace is True:
        return torch.zeros(plan.workspace_bytes // 4, dtype=torch.int32, device="cuda")
    return workspace


def deliver_slots(P, M, N, tile_m, tile_n, staging, part, flags, epoch, order, gap_us, side, n_wg, s16):
    """Peer slots through the emulated communicator; bf16 slots travel as fp32 pairs (N/2 columns, tile_n/2 per flag)."""
    if s16:
        pk.pk_emu_deliver_partials(P, M, N // 2, tile_m, tile_n // 2, staging, part, flags, epoch, order, gap_us,
                                   stream=side, n_wg=n_wg)
    else:
        pk.pk_emu_deliver_partials(P, M, N, tile_m, tile_n, staging, part, flags, epoch, order, gap_us, stream=side,
                                   n_wg=n_wg)


def run_gemm_rs(P, rank, M, N, K, dtype, A_bits, B_bits, partials, scale_a=None, scale_b=None,
                epoch=1, deliver="pre", order=None, gap_us=0, timeout_us=0, phases=pk.PHASE_ALL,
                withhold=None, lazy=False, partition=None, comm_cus=0, n_wg=0, partial_dtype="f32", cols=False,
                workspace=None, b_layout="kn"):
    """One pk_gemm_rs call.  b_layout = "nk": B_bits is the transposed matrix (N x K/P).  partials: numpy [P][M/P][N] fp32 (slot `rank` ignored).

    partition = (compute_stream, comm_stream) handles from pk_partition_create: the op then runs on the first and
    the emulated peers on the second.
    partial_dtype = "bf16": `partials` holds uint16 bit patterns; outgoing / partials_after come back as uint16.
    workspace: None, True (a fresh zeroed workspace of plan.workspace_bytes) or a device tensor to reuse.
    cols = True: pk_gemm_rs_cols (scatter along the last dimension): slots and the output are M x N/P.

    deliver = "pre": peer slots and their flags are in place before the call.
    deliver = "emu": peer slots start as NaN; pk_emu_deliver_partials copies them in on a second stream,
                     in `order`, with `gap_us` between slots, launched before the op.
    withhold: a (q, tile) whose flag is never set (timeout tests; "pre" only).
    Returns dict with out_bits (uint16), outgoing, partials_after, flags_out, flags_in, status, plan.
    lazy=True leaves the two big fp32 arrays on the device (keys outgoing_t, partials_t) instead.
    """
    plan = (pk.pk_gemm_rs_cols_plan if cols else pk.pk_gemm_rs_plan)(P, M, N, K, dtype)
    op = pk.pk_gemm_rs_cols if cols else pk.pk_gemm_rs
    # one shard is mp rows x ncols columns; the emulator sees [P][mp][ncols] slots of a (P*mp) x ncols problem
    mp = M if cols else M // P
    ncols = N // P if cols else N
    fps = plan.flags_per_slot
    A = elem_view(A_bits, dtype)
    B = elem_view(B_bits, dtype)
    sa, sb = scale_t(scale_a), scale_t(scale_b)
    out = torch.full((mp, ncols), -1, dtype=torch.int16, device="cuda")
    s16 = partial_dtype == "bf16"
    outgoing = slot_poison(P, mp, ncols, s16)
    flags_in = torch.zeros((P, fps), dtype=torch.int32, device="cuda")
    flags_out = torch.zeros((P, fps), dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    peers = [q for q in range(P) if q != rank]
    if order is None:
        order = peers
    main = torch.cuda.current_stream() if partition is None else torch.cuda.ExternalStream(partition[0])
    if deliver == "pre":
        part = slot_upload(partials, s16)
        part[rank].copy_(slot_poison(1, mp, ncols, s16)[0])
        for q in peers:
            flags_in[q].fill_(epoch)
        if withhold is not None:
            flags_in[withhold[0], withhold[1]] = epoch - 1
        torch.cuda.synchronize()
    else:
        staging = slot_upload(partials, s16)
        part = slot_poison(P, mp, ncols, s16)
        torch.cuda.synchronize()
        side = torch.cuda.Stream() if partition is None else torch.cuda.ExternalStream(partition[1])
        deliver_slots(P, P * mp, ncols, plan.tile_m, plan.tile_n, staging, part, flags_in, epoch, list(order), gap_us, side,
                      n_wg, s16)
    extra = {} if cols else {"workspace": make_workspace(plan, workspace), "b_layout": b_layout}
    op(P, rank, M, N, K, dtype, A, B, sa, sb, part, outgoing if P > 1 else None,
       flags_in, flags_out if P > 1 else None, epoch, out, phases, status, timeout_us, stream=main,
       comm_cus=comm_cus, partial_dtype=partial_dtype, **extra)
    torch.cuda.synchronize()
    res = {"out_bits": bits_of(out), "flags_out": flags_out.cpu().numpy(), "flags_in": flags_in.cpu().numpy(),
           "status": status.cpu().numpy(), "plan": plan}
    if lazy:
        res["outgoing_t"], res["partials_t"] = outgoing, part
    else:
        res["outgoing"], res["partials_after"] = slot_download(outgoing, s16), slot_download(part, s16)
    return res


def run_ag_gemm(P, rank, M, N, K, dtype, chunks, B_bits, scale_a=None, scale_b=None,
                epoch=1, deliver="pre", order=None, gap_us=0, timeout_us=0, withhold=None, fetch_A=True,
                comm_cus=0, n_wg=0, partition=None, act="none", workspace=None, b_layout="kn"):
    """One pk_ag_gemm call.  b_layout = "nk": B_bits is the transposed matrix (N/P x K).  chunks: list of P numpy bit arrays (M/P x K).

    deliver = "pre": every chunk is in A_gathered with its flag set before the call.
    deliver = "emu": only the own chunk is in place; the others are filled with a poison pattern and
                     pk_emu_deliver_chunks copies them in on a second stream in `order`.
    deliver = "dma": the same through pk_emu_deliver_chunks_dma (copies + stream flag writes, no workgroups).
    withhold: a chunk index whose flag is never set ("pre" only).
    """
    mp = M // P
    elem = 2 if dtype == "bf16" else 1
    npdt = np.uint16 if dtype == "bf16" else np.uint8
    poison = 0x7FC1 if dtype == "bf16" else 0x7F          # NaN patterns of the two formats
    B = elem_view(B_bits, dtype)
    sa, sb = scale_t(scale_a), scale_t(scale_b)
    C = torch.full((M, N // P), -1, dtype=torch.int16, device="cuda")
    flags = torch.zeros(P, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    peers = [q for q in range(P) if q != rank]
    if order is None:
        order = [(rank + d) % P for d in range(1, P)]
    main = torch.cuda.current_stream() if partition is None else torch.cuda.ExternalStream(partition[0])
    full = np.concatenate([np.asarray(c, dtype=npdt) for c in chunks], axis=0)
    if deliver == "pre":
        A = elem_view(full, dtype)
        for q in peers:
            flags[q] = epoch
        if withhold is not None:
            flags[withhold] = epoch - 1
        torch.cuda.synchronize()
    else:
        staging = elem_view(full, dtype)
        start = np.full_like(full, poison)
        start[rank * mp:(rank + 1) * mp] = full[rank * mp:(rank + 1) * mp]
        A = elem_view(start, dtype)
        counters = torch.zeros(pk.EMU_MAX_ORDER, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        side = torch.cuda.Stream() if partition is None else torch.cuda.ExternalStream(partition[1])
        if deliver == "dma":
            pk.pk_emu_deliver_chunks_dma(P, M, K, elem, staging, A, flags, epoch, list(order), stream=side)
        else:
            pk.pk_emu_deliver_chunks(P, M, K, elem, staging, A, flags, epoch, list(order), gap_us, counters, stream=side,
                                     n_wg=n_wg)
    ws = make_workspace(pk.pk_ag_gemm_plan(P, M, N, K, dtype), workspace)
    pk.pk_ag_gemm(P, rank, M, N, K, dtype, A, B, sa, sb, flags if P > 1 else None, epoch, C, status,
                  timeout_us, stream=main, comm_cus=comm_cus, act=act, workspace=ws, b_layout=b_layout)
    torch.cuda.synchronize()
    return {"C_bits": bits_of(C), "status": status.cpu().numpy(), "A_after": A.cpu().numpy() if fetch_A else None,
            "flags": flags.cpu().numpy()}


def run_gemm_ar(P, rank, M, N, K, dtype, A_bits, B_bits, partials, peer_rows, scale_a=None, scale_b=None, epoch=1,
                deliver="pre", order=None, gap_us=0, timeout_us=0, phases=pk.PHASE_ALL | pk.PHASE_WAIT,
                withhold_rows=None, partial_dtype="f32"):
    """One pk_gemm_ar call.  partials as run_gemm_rs; peer_rows: numpy [P][M/P][N] uint16, block q != rank is what
    rank q hands out for rows R_q of out_full.

    deliver = "pre": peers' partial slots and row blocks are in place with their flags set.
    deliver = "emu": both arrive through pk_emu_deliver_partials on a second stream (the bf16 rows as fp32 pairs),
                     into NaN-poisoned memory, partial slots first.
    withhold_rows: (q, flag index) of ar_flags_in never set ("pre" only).
    """
    plan = pk.pk_gemm_ar_plan(P, M, N, K, dtype)
    mp, fps, afps = M // P, plan.flags_per_slot, plan.ar_flags_per_slot
    A, B = elem_view(A_bits, dtype), elem_view(B_bits, dtype)
    sa, sb = scale_t(scale_a), scale_t(scale_b)
    poison_rows = np.full((P, mp, N), 0x7FC1, dtype=np.uint16)
    s16 = partial_dtype == "bf16"
    outgoing = slot_poison(P, mp, N, s16)
    bcast = dev(poison_rows.view(np.int16))
    flags_in = torch.zeros((P, fps), dtype=torch.int32, device="cuda")
    flags_out = torch.zeros((P, fps), dtype=torch.int32, device="cuda")
    ar_in = torch.zeros((P, afps), dtype=torch.int32, device="cuda")
    ar_out = torch.zeros((P, afps), dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    peers = [q for q in range(P) if q != rank]
    if order is None:
        order = peers
    main = torch.cuda.current_stream()
    peer_rows = np.ascontiguousarray(peer_rows, dtype=np.uint16)
    if deliver == "pre":
        part = slot_upload(partials, s16)
        part[rank].copy_(slot_poison(1, mp, N, s16)[0])
        start = peer_rows.copy()
        start[rank] = 0x7FC1
        full = dev(start.view(np.int16).reshape(M, N))
        for q in peers:
            flags_in[q].fill_(epoch)
            ar_in[q].fill_(epoch)
        if withhold_rows is not None:
            ar_in[withhold_rows[0], withhold_rows[1]] = epoch - 1
        torch.cuda.synchronize()
    else:
        staging = slot_upload(partials, s16)
        staging_rows = dev(peer_rows.view(np.int16))
        part = slot_poison(P, mp, N, s16)
        full = dev(poison_rows.view(np.int16).reshape(M, N))
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        deliver_slots(P, M, N, plan.tile_m, plan.tile_n, staging, part, flags_in, epoch, list(order), gap_us, side, 0, s16)
        # the bf16 row blocks as fp32 pairs: N/2 columns, PK_AR_ROWS x tile_n/2 per flag
        pk.pk_emu_deliver_partials(P, M, N // 2, pk.AR_ROWS, plan.tile_n // 2, staging_rows, full, ar_in, epoch,
                                   list(order), gap_us, stream=side)
    pk.pk_gemm_ar(P, rank, M, N, K, dtype, A, B, sa, sb, part, outgoing if P > 1 else None, flags_in,
                  flags_out if P > 1 else None, full, bcast if P > 1 else None, ar_in, ar_out if P > 1 else None, epoch,
                  phases, status, timeout_us, stream=main, partial_dtype=partial_dtype)
    torch.cuda.synchronize()
    return {"full_bits": bits_of(full), "bcast_bits": bits_of(bcast), "ar_in": ar_in.cpu().numpy(),
            "ar_out": ar_out.cpu().numpy(), "flags_out": flags_out.cpu().numpy(), "status": status.cpu().numpy(),
            "outgoing": slot_download(outgoing, s16), "plan": plan}


def run_ag_gemm_k(P, rank, M, N, K, dtype, chunks, B_bits, scale_a=None, scale_b=None, epoch=1, deliver="pre",
                  order=None, timeout_us=0, withhold=None, act="none"):
    """One pk_ag_gemm_k call.  chunks: list of P numpy bit arrays (M x K/P), chunk q = columns K_q of A.

    deliver = "pre": every chunk is in A_gathered with its flag set before the call.
    deliver = "dma": only the own chunk is in place, the others are poisoned; pk_emu_deliver_kchunks_dma copies them in on
                     a second stream in `order` (strided copies + stream flag writes).
    withhold: a chunk index whose flag is never set ("pre" only).
    """
    npdt = np.uint16 if dtype == "bf16" else np.uint8
    elem = 2 if dtype == "bf16" else 1
    poison = 0x7FC1 if dtype == "bf16" else 0x7F
    kp = K // P
    B = elem_view(B_bits, dtype)
    sa, sb = scale_t(scale_a), scale_t(scale_b)
    C = torch.full((M, N // P), -1, dtype=torch.int16, device="cuda")
    flags = torch.zeros(P, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    peers = [q for q in range(P) if q != rank]
    if order is None:
        order = [(rank + d) % P for d in range(1, P)]
    full = np.concatenate([np.asarray(c, dtype=npdt) for c in chunks], axis=1)
    main = torch.cuda.current_stream()
    if deliver == "pre":
        A = elem_view(full, dtype)
        for q in peers:
            flags[q] = epoch
        if withhold is not None:
            flags[withhold] = epoch - 1
        torch.cuda.synchronize()
    else:
        staging = elem_view(full, dtype)
        start = np.full_like(full, poison)
        start[:, rank * kp:(rank + 1) * kp] = full[:, rank * kp:(rank + 1) * kp]
        A = elem_view(start, dtype)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        pk.pk_emu_deliver_kchunks_dma(P, M, K, elem, staging, A, flags, epoch, list(order), stream=side)
    pk.pk_ag_gemm_k(P, rank, M, N, K, dtype, A, B, sa, sb, flags if P > 1 else None, epoch, C, status, timeout_us,
                    stream=main, act=act)
    torch.cuda.synchronize()
    return {"C_bits": bits_of(C), "status": status.cpu().numpy(), "A_after": A.cpu().numpy(), "flags": flags.cpu().numpy()}
