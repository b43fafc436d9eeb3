#!/usr/bin/env python3
"""Benchmark of the per-rank tensor-parallel hot path on one MI355X.

One step = one pass over the MLP share of a 70B-class model under 8-way tensor parallelism:
  pk_ag_gemm  (cfg4: A gathered from 8 chunks of 1024 x 8192, B_local 8192 x 3584)   -> tile schedule,
              per-chunk flag wait, MFMA main loop, bf16 epilogue
  pk_gemm_rs  (cfg3: A_local 8192 x 3584, B_local 3584 x 8192, 7 peer partials)      -> tile schedule, MFMA
              main loop, fp32 scatter epilogue + per-tile signal, fused reduce of the 8 partial slots
with every input (operands, the peers' chunks and partial sums, their ready flags) resident in HBM when the
timed region starts.  The metric is the paper's "observed average compute throughput": flops of the two
local GEMMs divided by the time of the step.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}      # MI355X dense MFMA peak
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing / parity leg")
    ap.add_argument("--preheat-ms", type=float, default=150.0,
                    help="untimed sustained run of the same step before the warm-up steps: the clock governor needs "
                         "~70 ms of load to settle (0 = measure the cold-start transient instead)")
    ap.add_argument("--extras", action="store_true", help="also time the phases alone and the live-arrival variants")
    ap.add_argument("--buffer-sets", type=int, default=3,
                    help="copies of every operand, partial-slot and output buffer that the timed steps rotate through")
    ap.add_argument("--serial-reduce", action="store_true",
                    help="run the reduce of GEMM+RS after its GEMM instead of beside it (no PK_PHASE_OVERLAP)")
    ap.add_argument("--only-step", action="store_true",
                    help="time the step and nothing else (for profiler runs: no other launches of the same kernels)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one rank's share on ONE GPU (peers are emulated in the same HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_13940_amd import pk, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    pk.lib()                                            # fail loudly if the HIP library is missing
    rank = 0
    c3, c4 = wl.CONFIGS["cfg3"], wl.CONFIGS["cfg4"]
    RS_PHASES = pk.PHASE_ALL | (0 if args.serial_reduce else pk.PHASE_OVERLAP)

    # ---------------- inputs (seeded, synthetic), uploaded once ----------------
    t0 = time.time()
    i3 = wl.gemm_rs_inputs(c3.P, c3.M, c3.N, c3.K, c3.dtype, rank, seed=0, order=c3.order)
    i4 = wl.ag_gemm_inputs(c4.P, c4.M, c4.N, c4.K, c4.dtype, rank, seed=0, order=c4.order)
    a4_full = np.concatenate(i4["chunks"], axis=0)
    gen_s = time.time() - t0

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x)).cuda()

    p3 = pk.pk_gemm_rs_plan(c3.P, c3.M, c3.N, c3.K, c3.dtype)
    mp3 = c3.M // c3.P
    A3, B3 = dev(i3["A_local"].view(np.int16)), dev(i3["B_local"].view(np.int16))
    part = dev(i3["partials"])
    outgoing = torch.zeros((c3.P, mp3, c3.N), dtype=torch.float32, device="cuda")
    out3 = torch.zeros((mp3, c3.N), dtype=torch.int16, device="cuda")
    flags_in = torch.zeros((c3.P, p3.flags_per_slot), dtype=torch.int32, device="cuda")
    flags_out = torch.zeros_like(flags_in)
    for q in range(c3.P):
        if q != rank:
            flags_in[q].fill_(0x7FFFFFFF)               # peers' partials are resident: ready for every epoch
    A4, B4 = dev(a4_full.view(np.int16)), dev(i4["B_local"].view(np.int16))
    C4 = torch.zeros((c4.M, c4.N // c4.P), dtype=torch.int16, device="cuda")
    chunk_flags = torch.full((c4.P,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    status = torch.zeros(8, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    # Buffer sets the steps rotate through (step e uses set e mod n), so that no step finds its operands, slots or outputs
    # where the same step left them: set 0 is the tensors above, the others are copies (about 1 GB each, four times the
    # 256 MB Infinity Cache already).
    names = ("A3", "B3", "part", "outgoing", "out3", "flags_in", "flags_out", "A4", "B4", "C4")
    here = locals()
    sets = [{k: here[k] for k in names}]
    for _ in range(max(args.buffer_sets, 1) - 1):
        sets.append({k: v.clone() for k, v in sets[0].items()})

    def step(epoch, ev=None):
        # the timed step: AG+GEMM, then GEMM+RS with its reduce hidden behind the GEMM (one call, PK_PHASE_OVERLAP)
        S = sets[epoch % len(sets)]
        if ev:
            ev[0].record(stream)
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, S["A4"], S["B4"], None, None, chunk_flags, epoch, S["C4"], status)
        if ev:
            ev[1].record(stream)
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, S["A3"], S["B3"], None, None, S["part"], S["outgoing"],
                      S["flags_in"], S["flags_out"], epoch, S["out3"], RS_PHASES, status)

    def step_serial(epoch, ev=None):
        # the same step with the two phases of GEMM+RS as calls of their own, one after the other.  ev: 2 events (around
        # the cfg4 launch, like the timed step) or 4 (a third and fourth behind the cfg3 GEMM and the reduce: durations)
        S = sets[epoch % len(sets)]
        if ev:
            ev[0].record(stream)
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, S["A4"], S["B4"], None, None, chunk_flags, epoch, S["C4"], status)
        if ev:
            ev[1].record(stream)
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, S["A3"], S["B3"], None, None, S["part"], S["outgoing"],
                      S["flags_in"], S["flags_out"], epoch, S["out3"], pk.PHASE_GEMM, status)
        if ev and len(ev) > 2:
            ev[2].record(stream)
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, None, None, None, None, S["part"], None,
                      S["flags_in"], None, epoch, S["out3"], pk.PHASE_REDUCE, status)
        if ev and len(ev) > 2:
            ev[3].record(stream)

    # a plain copy of known size (64 MiB read + 64 MiB written): the yardstick for HBM-traffic counters
    cal_src = torch.ones(16 * 1024 * 1024, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)

    epoch = 0
    # The chip's clock governor answers a load that starts from idle by dropping the core clock and raising it again
    # over ~50-70 ms (measured: the same launch takes 0.47 ms 4 ms after the start and 0.36 ms from 70 ms on).  A
    # deployment runs these kernels back to back, so the step is timed in that settled state: the preheat below is
    # the same step, untimed, for --preheat-ms of GPU time.  The first timed-order steps from idle are reported too.
    epoch += 1
    step(epoch)                                        # loads the code objects; not part of any timing
    torch.cuda.synchronize()
    time.sleep(0.2)
    cold = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    cold[0].record(stream)
    for _ in range(5):
        epoch += 1
        step(epoch)
    cold[1].record(stream)
    torch.cuda.synchronize()
    cold_ms = cold[0].elapsed_time(cold[1]) / 5
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.preheat_ms:
        for _ in range(20):
            epoch += 1
            step(epoch)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        epoch += 1
        step(epoch)
    # two events per timed step, around the cfg4 launch (an event record costs the stream 3-5 us)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    ev_end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        epoch += 1
        step(epoch, evs[i])
    ev_end.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert status[0].item() == 0, f"device status {status.tolist()}"

    ms_step = wall * 1e3 / args.steps
    per_ag = [e[0].elapsed_time(e[1]) for e in evs]
    per_rs_op = [evs[i][1].elapsed_time(evs[i + 1][0] if i + 1 < args.steps else ev_end) for i in range(args.steps)]
    k_ag, op_rs = sum(per_ag) / args.steps, sum(per_rs_op) / args.steps   # the cfg4 GEMM launch; the whole GEMM+RS call

    # the same number of steps with the phases of GEMM+RS apart (not part of `value`), with the same two events per step
    evs_s = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        epoch += 1
        step_serial(epoch, evs_s[i])
    torch.cuda.synchronize()
    ms_step_serial = (time.perf_counter() - t0) * 1e3 / args.steps
    # and once more with an event behind every launch: the cfg3 GEMM as one launch, the reduce kernel alone behind it
    evs_s = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
        epoch += 1
        step_serial(epoch, evs_s[i])
    torch.cuda.synchronize()
    assert status[0].item() == 0, f"device status {status.tolist()}"
    st_words = [x & 0xFFFFFFFF for x in status.tolist()]      # timing report of the last GEMM launch (the cfg3 one)
    per = [[e[i].elapsed_time(e[i + 1]) for e in evs_s] for i in range(3)]
    k_ag_serial, k_rs, k_red = (sum(x) / args.steps for x in per)
    per[0] = per_ag                                           # the cfg4 kernel's durations come from the timed steps

    # and once more on one buffer set only (every step finds what the Infinity Cache kept of the step before): cache-warm
    ms_step_one_set = None
    if len(sets) > 1 and not args.only_step:
        rotating, sets = sets, sets[:1]
        for _ in range(args.warmup):
            epoch += 1
            step(epoch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            epoch += 1
            step(epoch)
        torch.cuda.synchronize()
        ms_step_one_set = (time.perf_counter() - t0) * 1e3 / args.steps
        sets = rotating
        del rotating
    sets = sets[:1]                                           # the copies are not needed any more

    # the MFMA rate this chip sustains in a register-only loop: operands all 1.0, then random sign + mantissa
    # (data-dependent power lowers the clock); per-run context for the roofline fraction below
    report = torch.zeros(4, dtype=torch.int64, device="cuda")
    sustained = {}
    for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
        if args.only_step:
            break
        pk.pk_probe_mfma(2000, rnd, report)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fl = pk.pk_probe_mfma(20000, rnd, report)
        b.record(stream)
        torch.cuda.synchronize()
        rep = report.tolist()
        sustained[label] = {"TFLOP/s": round(fl / (a.elapsed_time(b) * 1e-3) / 1e12, 1),
                            "core_clock_MHz": round(100.0 * rep[1] / max(rep[0], 1))}
    flops = c3.flops + c4.flops
    value = flops / (ms_step * 1e-3) / 1e12

    # ---------------- roofline of the dominant kernel ----------------
    red_bytes = c3.M * c3.N * 4 + mp3 * c3.N * 2           # P slots of fp32 read + bf16 shard written
    kernels = {
        "gemm_kernel<256,256,bf16,AG> (cfg4)": {"ms": k_ag, "TFLOP/s": c4.flops / (k_ag * 1e-3) / 1e12},
        "gemm_kernel<256,256,bf16,RS> (cfg3)": {"ms": k_rs, "TFLOP/s": c3.flops / (k_rs * 1e-3) / 1e12},
        "reduce_kernel<8> (cfg3)": {"ms": k_red, "GB/s": red_bytes / (k_red * 1e-3) / 1e9},
    }
    # the kernel the roofline is quoted for is the cfg4 GEMM: one launch per timed step, bracketed by events there (the
    # cfg3 GEMM runs as two launches beside the reduce in the timed steps; its single-launch duration is the serial one)
    dom = "gemm_kernel<256,256,bf16,AG> (cfg4)"
    ach = kernels[dom]["TFLOP/s"]
    traffic = measured_traffic()
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(ach, 2), "peak": PEAK_TFLOPS["bf16"],
                "unit": "TFLOP/s", "frac": round(ach / PEAK_TFLOPS["bf16"], 4), "traffic": traffic.get(dom),
                "traffic_unit": "bytes beyond L2 per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, see profiles/)",
                "kernel_ms": round(kernels[dom]["ms"], 4),
                "traffic_source": "profiles/bench_step_hbm_traffic.txt (measured offline with rocprofv3 --pmc on the commit "
                                  "named in that file; not re-measured by this run)",
                "mfma_loop_sustained": sustained,
                "frac_of_sustained_random": round(ach / sustained["random_operands"]["TFLOP/s"], 4) if sustained else None}
    reduce_roofline = {"bound": "hbm", "kernel": "reduce_kernel<8> (cfg3)",
                       "achieved": round(kernels["reduce_kernel<8> (cfg3)"]["GB/s"], 1), "peak": PEAK_HBM_GBS,
                       "unit": "GB/s", "frac": round(kernels["reduce_kernel<8> (cfg3)"]["GB/s"] / PEAK_HBM_GBS, 4),
                       "traffic": traffic.get("reduce_kernel<8> (cfg3)"), "algorithmic_bytes": red_bytes,
                       "kernel_ms": round(k_red, 4)}

    result = {
        "metric": "per-rank TFLOP/s (GEMM+RS, AG+GEMM) and % of MFMA/HBM roofline, 1 MI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg4 AG+GEMM (P=8, A 8x[1024x8192], B_local 8192x3584) + cfg3 GEMM+RS "
                               "(P=8, A_local 8192x3584, B_local 3584x8192, 7 fp32 peer partials 1024x8192); "
                               "70B-MLP TP=8 share, rank 0, peers' data pre-landed with flags set",
                   "flops_per_step": flops},
        "roofline": roofline,
        "reduce_roofline": reduce_roofline,
        "kernels": {k: {kk: round(vv, 4) for kk, vv in v.items()} for k, v in kernels.items()},
        "kernel_ms_median_min": {k: [round(sorted(x)[len(x) // 2], 4), round(min(x), 4)]
                                 for k, x in zip(kernels, per)},
        "frac_of_mfma_peak_whole_step": round(value / PEAK_TFLOPS["bf16"], 4),
        "gemm_rs_call_ms_in_timed_steps": round(op_rs, 4),
        "reduce_overlapped": bool(RS_PHASES & pk.PHASE_OVERLAP),
        "ms_per_step_with_serial_reduce": round(ms_step_serial, 4),
        "TFLOP/s_with_serial_reduce": round(flops / (ms_step_serial * 1e-3) / 1e12, 2),
        "preheat_ms": args.preheat_ms,
        "buffer_sets_rotated": max(args.buffer_sets, 1),
        "ms_per_step_one_buffer_set_cache_warm": round(ms_step_one_set, 4) if ms_step_one_set else None,
        "ms_per_step_first_5_steps_from_idle": round(cold_ms, 4),
        "in_kernel_clock_report_cfg3_gemm": {
            "core_clock_MHz": round(100.0 * st_words[5] / max(st_words[4], 1)),
            "main_loop_share_of_cycles": round(st_words[6] / max(st_words[5], 1), 4),
            "mfma_issue_share_inside_main_loops": round(32.0 * (c3.K // c3.P) * st_words[7] / max(st_words[6], 1), 4)},
    }

    if not args.only_step:
        result.update(more_measurements(pk, wl, torch, np, locals()))
        result["diagnosis"] = diagnosis(pk, torch, locals())
    if args.extras:
        result["extras"] = extras(pk, wl, torch, np, locals())

    # ---------------- CPU baseline: the oracle as it stands, and parity of this run's outputs ----------------
    if not args.no_cpu_baseline:
        from oracle import codec, tp_gemm
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        rows3 = np.arange(0, c3.M)                      # the whole workload: the oracle takes seconds here
        rows4 = np.arange(0, c4.M)
        t0 = time.perf_counter()
        own_rows, out_rows = tp_gemm.gemm_rs_rows(c3.P, rank, i3["A_local"], i3["B_local"], c3.dtype,
                                                  i3["partials"], rows3)
        c_rows = tp_gemm.ag_gemm(c4.P, rank, a4_full, i4["B_local"], c4.dtype, rows=rows4)["C"]
        cpu_s = time.perf_counter() - t0
        sample_flops = 2 * len(rows3) * c3.N * (c3.K // c3.P) + 2 * len(rows4) * (c4.N // c4.P) * c4.K
        result["cpu_baseline"] = {"value": round(sample_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores),
                                  "kind": "oracle", "seconds": round(cpu_s, 2),
                                  "sample": "the whole step: both local GEMMs in full (8192 rows each, all columns, full K) "
                                            "plus the 8-slot reduce of the own shard"}
        # parity of the benchmarked buffers on the sampled rows
        gate = lambda g, r: float(np.max(np.abs(g - r) / (np.abs(r) + 1.0)))
        own_rank_rows = rows3[rows3 // mp3 == rank]
        got3 = codec.bf16_decode(out3.cpu().numpy().view(np.uint16))[own_rank_rows - rank * mp3]
        ref3 = out_rows[rows3 // mp3 == rank]
        got4 = codec.bf16_decode(C4.cpu().numpy().view(np.uint16))[rows4]
        og = outgoing.cpu().numpy()
        scat_err = 0.0
        for q in range(c3.P):
            if q == rank:
                continue
            sel = rows3 // mp3 == q
            scat_err = max(scat_err, gate(og[q][rows3[sel] - q * mp3], own_rows[sel]))
        # beside the gate: the largest error against the rms of the reference, and the share of outputs within one bf16
        # unit in the last place of the correctly rounded reference (inputs ~N(0,1)/sqrt(K) make |ref| << 1, so the gate
        # alone is an absolute 1e-2)
        def ulp_stats(g, r):
            rb = codec.bf16_decode(codec.bf16_encode(r))
            ulp = np.maximum(np.abs(rb), 2.0 ** -126) * 2.0 ** -7
            return {"max_abs_err_over_rms_ref": float(np.max(np.abs(g - r)) / np.sqrt(np.mean(r * r))),
                    "share_within_1_bf16_ulp_of_rounded_ref": float(np.mean(np.abs(g - rb) <= ulp))}
        result["parity"] = {"metric": "max|gpu-ref|/(|ref|+1) on the sampled rows", "gemm_rs_out": gate(got3, ref3),
                            "gemm_rs_outgoing": scat_err, "ag_gemm_C": gate(got4, c_rows), "tolerance": 1e-2,
                            "gemm_rs_out_detail": ulp_stats(got3, ref3), "ag_gemm_C_detail": ulp_stats(got4, c_rows)}
        assert max(result["parity"]["gemm_rs_out"], scat_err, result["parity"]["ag_gemm_C"]) <= 1e-2, result["parity"]

    result["setup_seconds"] = round(gen_s, 1)
    print(json.dumps(result))


def measured_traffic():
    """HBM-side traffic per launch of the step's kernels, as measured by the committed rocprofv3 counter runs
    (bench.py cannot run the profiler on itself).  Returns {kernel label: bytes} or {} if the summary is absent."""
    path = os.path.join(ROOT, "profiles", "bench_step_hbm_traffic.txt")
    out = {}
    try:
        with open(path) as f:
            for ln in f:
                if ln.startswith("TRAFFIC|"):
                    _, label, fetch, write = ln.strip().split("|")
                    out[label] = int(fetch) + int(write)
    except OSError:
        pass
    return out


def _timeit(torch, stream, fn, n=20, w=5, st=None):
    st = st or stream
    for _ in range(w):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(st)
    for _ in range(n):
        fn()
    b.record(st)
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


def more_measurements(pk, wl, torch, np, L):
    """The other figures of the measurement plan, all in the settled clock state: the Table-3-style pair for cfg3 (bare
    GEMM against the fused op), cfg5 (fp8, HBM-bound) with its own roofline, the live-arrival cases on a compute-unit
    partition, and the gather phase alone."""
    c3, c4, rank, stream, status = L["c3"], L["c4"], L["rank"], L["stream"], L["status"]
    out = {}
    timeit = lambda fn, n=20, w=5, st=None: _timeit(torch, stream, fn, n, w, st)
    ep = [20 * 10 ** 6]

    # --- cfg3: GEMM alone (same kernel, bf16 output, no flags) against GEMM + reduce-scatter, as the paper's Table 3 ---
    m, n, k = c3.local_mnk
    Cg = torch.zeros((m, n), dtype=torch.int16, device="cuda")
    t_gemm = timeit(lambda: pk.pk_ag_gemm(1, 0, m, n, k, "bf16", L["A3"], L["B3"], None, None, None, 1, Cg, status), w=30)

    def fused(phases):
        def f():
            ep[0] += 1
            pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                          L["flags_in"], L["flags_out"], ep[0], L["out3"], phases, status)
        return f
    t_serial = timeit(fused(pk.PHASE_ALL), w=30)
    t_fused = timeit(fused(pk.PHASE_ALL | pk.PHASE_OVERLAP), w=30)
    out["table3_style_cfg3"] = {"t_gemm_ms": round(t_gemm, 4), "t_fused_ms": round(t_fused, 4),
                                "comm_ratio": round((t_fused - t_gemm) / t_fused, 4),
                                "gemm_TFLOP/s": round(c3.flops / (t_gemm * 1e-3) / 1e12, 1),
                                "fused_TFLOP/s": round(c3.flops / (t_fused * 1e-3) / 1e12, 1),
                                "t_fused_serial_reduce_ms": round(t_serial, 4),
                                "comm_ratio_serial_reduce": round((t_serial - t_gemm) / t_serial, 4)}
    # the same with bf16 partial slots (the paper's element size for communicated tiles, s = 2 in its cost model)
    part16 = L["part"].to(torch.bfloat16).view(torch.int16)
    outg16 = torch.empty(part16.shape, dtype=torch.int16, device="cuda")

    def fused16(phases):
        def f():
            ep[0] += 1
            pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, part16, outg16,
                          L["flags_in"], L["flags_out"], ep[0], L["out3"], phases, status, partial_dtype="bf16")
        return f
    t16s = timeit(fused16(pk.PHASE_ALL), w=30)
    t16 = timeit(fused16(pk.PHASE_ALL | pk.PHASE_OVERLAP), w=30)
    out["table3_style_cfg3"]["bf16_partial_slots"] = {
        "t_fused_ms": round(t16, 4), "comm_ratio": round((t16 - t_gemm) / t16, 4),
        "fused_TFLOP/s": round(c3.flops / (t16 * 1e-3) / 1e12, 1),
        "t_fused_serial_reduce_ms": round(t16s, 4), "comm_ratio_serial_reduce": round((t16s - t_gemm) / t16s, 4)}
    fused(pk.PHASE_ALL | pk.PHASE_OVERLAP)()          # leaves the fp32-slot result in out3 for the parity check of this run
    del part16, outg16
    del Cg

    # --- variants of the two GEMM kernels, each timed alone back to back on the same buffers ---
    plan4 = pk.pk_ag_gemm_plan(c4.P, c4.M, c4.N, c4.K, c4.dtype)
    ws = torch.zeros(plan4.workspace_bytes // 4, dtype=torch.int32, device="cuda")
    B4t, B3t = L["B4"].t().contiguous(), L["B3"].t().contiguous()

    def ag(**kw):
        def f():
            ep[0] += 1
            pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], kw.get("B", L["B4"]),
                          None, None, L["chunk_flags"], ep[0], L["C4"], status, workspace=kw.get("workspace"),
                          b_layout=kw.get("b_layout", "kn"))
        return f

    def rsg(**kw):
        def f():
            ep[0] += 1
            pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], kw.get("B", L["B3"]), None, None, L["part"],
                          L["outgoing"], L["flags_in"], L["flags_out"], ep[0], L["out3"], pk.PHASE_GEMM, status,
                          b_layout=kw.get("b_layout", "kn"))
        return f
    t_ag, t_ag_sk, t_ag_bt = timeit(ag(), n=60, w=40), timeit(ag(workspace=ws), n=60, w=40), timeit(ag(B=B4t, b_layout="nk"), n=60, w=40)
    t_rs, t_rs_bt = timeit(rsg(), n=60, w=40), timeit(rsg(B=B3t, b_layout="nk"), n=60, w=40)
    out["kernel_variants_alone_ms"] = {
        "ag_gemm_cfg4": {"whole_tiles_224_workgroups": round(t_ag, 4), "stream_k_tail_256_workgroups": round(t_ag_sk, 4),
                         "b_k_contiguous": round(t_ag_bt, 4)},
        "gemm_rs_cfg3_gemm_phase": {"b_row_major": round(t_rs, 4), "b_k_contiguous": round(t_rs_bt, 4)}}
    del ws, B4t, B3t

    # --- gather phase alone: the emulated communicator moving the 7 peer chunks of cfg4 with 256 workgroups ---
    staging = L["A4"].clone()
    counters = torch.zeros(pk.EMU_MAX_ORDER, dtype=torch.int32, device="cuda")
    order = L["i4"]["order"]
    moved = 2 * (c4.P - 1) * (c4.M // c4.P) * c4.K * 2

    def gather():
        counters.zero_()
        pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], L["chunk_flags"], 0x7FFFFFFF, order, 0, counters, n_wg=256)
    t_g = timeit(gather)
    out["gather_phase_cfg4"] = {"ms": round(t_g, 4), "GB/s": round(moved / (t_g * 1e-3) / 1e9, 1),
                                "frac_of_hbm_peak": round(moved / (t_g * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "workgroups": 256}

    # --- live arrival on a compute-unit partition (communicator on COMM compute units, the op on the others) ---
    COMM = 32
    h_comp, h_comm = pk.pk_partition_create(COMM)
    comp, side = torch.cuda.ExternalStream(h_comp), torch.cuda.ExternalStream(h_comm)
    flags_live = torch.zeros(c4.P, dtype=torch.int32, device="cuda")
    done = torch.cuda.Event()
    torch.cuda.synchronize()

    def ag_live():
        ep[0] += 1
        done.record(comp)
        side.wait_event(done)
        with torch.cuda.stream(side):
            counters.zero_()
        pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_live, ep[0], order, 0, counters,
                                 stream=side, n_wg=8 * COMM)
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, flags_live, ep[0], L["C4"],
                      status, comm_cus=COMM, stream=comp)
        comp.wait_stream(side)
    t_ag_live = timeit(ag_live, w=30, st=comp)
    t_ag_pre = timeit(lambda: pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None,
                                            L["chunk_flags"], 1, L["C4"], status, comm_cus=COMM, stream=comp), st=comp)
    flags_live3 = torch.zeros_like(L["flags_in"])
    stage3 = L["part"].clone()
    p3 = L["p3"]
    peers = [q for q in range(c3.P) if q != rank]

    def rs_live():
        ep[0] += 1
        done.record(comp)
        side.wait_event(done)
        pk.pk_emu_deliver_partials(c3.P, c3.M, c3.N, p3.tile_m, p3.tile_n, stage3, L["part"], flags_live3, ep[0],
                                   peers, 0, stream=side, n_wg=8 * COMM)
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                      flags_live3, L["flags_out"], ep[0], L["out3"], pk.PHASE_ALL, status, comm_cus=COMM, stream=comp)
        comp.wait_stream(side)
    t_rs_live = timeit(rs_live, w=30, st=comp)

    def rs_pre():
        ep[0] += 1
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                      L["flags_in"], L["flags_out"], ep[0], L["out3"], pk.PHASE_ALL, status, comm_cus=COMM, stream=comp)
    t_rs_pre = timeit(rs_pre, st=comp)
    torch.cuda.synchronize()
    pk.pk_partition_destroy(h_comp, h_comm)

    # --- live arrival without a partition: the op on every compute unit, the communicator's workgroups (no LDS, under 64
    # registers) resident beside the GEMM's on the same compute units, on a second stream ---
    side2 = torch.cuda.Stream()

    def ag_live_beside():
        ep[0] += 1
        done.record(stream)
        side2.wait_event(done)
        with torch.cuda.stream(side2):
            counters.zero_()
        pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_live, ep[0], order, 0, counters,
                                 stream=side2, n_wg=256)
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, flags_live, ep[0], L["C4"], status)
        stream.wait_stream(side2)
    t_ag_beside = timeit(ag_live_beside, w=30)      # (a longer warm-up: this mix of kernels settles at its own clock)
    t_ag_pre_all = timeit(lambda: pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None,
                                                L["chunk_flags"], 1, L["C4"], status))

    def rs_live_beside():
        ep[0] += 1
        done.record(stream)
        side2.wait_event(done)
        pk.pk_emu_deliver_partials(c3.P, c3.M, c3.N, p3.tile_m, p3.tile_n, stage3, L["part"], flags_live3, ep[0],
                                   peers, 0, stream=side2, n_wg=512)
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                      flags_live3, L["flags_out"], ep[0], L["out3"], pk.PHASE_ALL, status)
        stream.wait_stream(side2)
    t_rs_beside = timeit(rs_live_beside, w=30)
    out["live_arrival_no_partition"] = {
        "ag_gemm_cfg4": {"t_fused_live_ms": round(t_ag_beside, 4), "t_fused_prelanded_ms": round(t_ag_pre_all, 4),
                         "live_over_prelanded": round(t_ag_beside / t_ag_pre_all, 3), "communicator_workgroups": 256},
        "gemm_rs_cfg3": {"t_fused_live_ms": round(t_rs_beside, 4), "t_fused_prelanded_ms": round(t_serial, 4),
                         "live_over_prelanded": round(t_rs_beside / t_serial, 3), "communicator_workgroups": 512}}
    out["live_arrival"] = {
        "comm_cus": COMM,
        "ag_gemm_cfg4": {"t_fused_live_ms": round(t_ag_live, 4), "t_fused_prelanded_same_partition_ms": round(t_ag_pre, 4),
                         "live_over_prelanded": round(t_ag_live / t_ag_pre, 3)},
        "gemm_rs_cfg3": {"t_fused_live_ms": round(t_rs_live, 4), "t_fused_prelanded_same_partition_ms": round(t_rs_pre, 4),
                         "live_over_prelanded": round(t_rs_live / t_rs_pre, 3)}}
    del staging, stage3

    # --- cfg5: fp8 e4m3 GEMM + reduce-scatter; HBM-bound (2.28 GB of mandatory traffic for 1.1e12 flop) ---
    c5 = wl.CONFIGS["cfg5"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(251113945)
    p5 = pk.pk_gemm_rs_plan(c5.P, c5.M, c5.N, c5.K, c5.dtype)
    mp5, k5 = c5.M // c5.P, c5.K // c5.P
    # operands: N(0,1)/sqrt(K) quantised to e4m3 with a per-tensor scale amax/448 (drawn on the device: parity of this
    # configuration is the tests' business); peer partials N(0, sigma_p^2) as in the recipe
    def q8(rows, cols):
        x = torch.randn((rows, cols), generator=gen, device="cuda") / c5.K ** 0.5
        sc = x.abs().max() / 448.0
        return (x / sc).to(torch.float8_e4m3fn).view(torch.uint8), sc.reshape(1).float()
    A5, sa5 = q8(c5.M, k5)
    B5, sb5 = q8(k5, c5.N)
    part5 = torch.randn((c5.P, mp5, c5.N), generator=gen, device="cuda") * (k5 ** 0.5 / c5.K)
    outg5 = torch.zeros((c5.P, mp5, c5.N), dtype=torch.float32, device="cuda")
    out5 = torch.zeros((mp5, c5.N), dtype=torch.int16, device="cuda")
    fin5 = torch.full((c5.P, p5.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    fin5[rank].zero_()
    fout5 = torch.zeros_like(fin5)

    def rs5(phases):
        def f():
            if phases & 1:
                ep[0] += 1
            pk.pk_gemm_rs(c5.P, rank, c5.M, c5.N, c5.K, c5.dtype, A5, B5, sa5, sb5, part5, outg5, fin5, fout5, ep[0], out5,
                          phases, status)
        return f
    t5s = timeit(rs5(pk.PHASE_ALL), n=10, w=20)
    t5 = timeit(rs5(pk.PHASE_ALL | pk.PHASE_OVERLAP), n=10, w=20)
    t5g = timeit(rs5(pk.PHASE_GEMM), n=10, w=20)
    t5r = timeit(rs5(pk.PHASE_REDUCE), n=10, w=20)
    bytes5 = 2 * c5.M * k5 + 2 * c5.M * c5.N * 4 + mp5 * c5.N * 2
    red5 = c5.M * c5.N * 4 + mp5 * c5.N * 2
    out["cfg5_fp8_gemm_rs"] = {
        "ms": round(t5, 4), "TFLOP/s": round(c5.flops / (t5 * 1e-3) / 1e12, 1),
        "roofline": {"bound": "hbm", "achieved": round(bytes5 / (t5 * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(bytes5 / (t5 * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "algorithmic_bytes": bytes5, "traffic": None},
        "ms_serial_reduce": round(t5s, 4),
        "gemm_phase_ms": round(t5g, 4), "gemm_phase_TFLOP/s": round(c5.flops / (t5g * 1e-3) / 1e12, 1),
        "gemm_phase_frac_of_fp8_mfma_peak": round(c5.flops / (t5g * 1e-3) / 1e12 / PEAK_TFLOPS["fp8"], 4),
        "reduce_phase_ms": round(t5r, 4), "reduce_phase_GB/s": round(red5 / (t5r * 1e-3) / 1e9, 1)}
    # the same op with bf16 partial slots (the paper's element size for communicated tiles, s = 2): half the scatter and reduce traffic
    part16 = part5.to(torch.bfloat16).view(torch.int16)
    del part5
    outg16 = outg5.view(torch.int16).reshape(-1)[:c5.P * mp5 * c5.N].view(c5.P, mp5, c5.N)

    def rs5_16(phases):
        def f():
            if phases & 1:
                ep[0] += 1
            pk.pk_gemm_rs(c5.P, rank, c5.M, c5.N, c5.K, c5.dtype, A5, B5, sa5, sb5, part16, outg16, fin5, fout5, ep[0], out5,
                          phases, status, partial_dtype="bf16")
        return f
    t16 = timeit(rs5_16(pk.PHASE_ALL | pk.PHASE_OVERLAP), n=10, w=20)   # (next to the fp8 kernel: falls back to the serial reduce)
    t16g = timeit(rs5_16(pk.PHASE_GEMM), n=10, w=20)
    t16r = timeit(rs5_16(pk.PHASE_REDUCE), n=10, w=20)
    bytes16 = 2 * c5.M * k5 + 2 * c5.M * c5.N * 2 + mp5 * c5.N * 2
    out["cfg5_fp8_gemm_rs"]["bf16_partial_slots"] = {
        "ms": round(t16, 4), "TFLOP/s": round(c5.flops / (t16 * 1e-3) / 1e12, 1), "gemm_phase_ms": round(t16g, 4),
        "reduce_phase_ms": round(t16r, 4), "algorithmic_bytes": bytes16,
        "frac_of_hbm_peak_on_its_own_bytes": round(bytes16 / (t16 * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    assert status[0].item() == 0, f"device status {status.tolist()}"
    return out


def diagnosis(pk, torch, L):
    """What holds the bf16 GEMM below the MFMA peak, measured through the product entry point (a bare GEMM of the cfg3
    local shape, 4 tiles of 256 x 256 x 3584 per workgroup) with the kernel's own clock report: the core clock the chip
    holds as a function of (a) how many compute units are busy, (b) the bit activity of the operands, (c) the time since
    the load began.  The instruction schedule is the same in every row."""
    stream, status = L["stream"], L["status"]
    n, k = 8192, 3584
    A, B = L["A3"], L["B3"]                      # 8192 x 3584 and 3584 x 8192, N(0,1)/sqrt(K) in bf16
    C = torch.zeros((8192, n), dtype=torch.int16, device="cuda")

    def run(m, comm, a, b, reps=150):
        fn = lambda: pk.pk_ag_gemm(1, 0, m, n, k, "bf16", a, b, None, None, None, 1, C, status, comm_cus=comm)
        ms = _timeit(torch, stream, fn, n=reps, w=reps)
        st = [x & 0xFFFFFFFF for x in status.tolist()]
        return {"ms": round(ms, 4), "TFLOP/s": round(2.0 * m * n * k / (ms * 1e-3) / 1e12, 1),
                "core_clock_MHz": round(100.0 * st[5] / max(st[4], 1)),
                "mfma_issue_share_in_main_loops": round(32.0 * k * st[7] / max(st[6], 1), 3),
                "main_loop_share_of_cycles": round(st[6] / max(st[5], 1), 3)}
    out = {"kernel": "gemm_kernel<256,256,bf16> as a bare GEMM, n = 8192, k = 3584, m = 32 rows per workgroup x 4 tiles",
           "active_compute_units": {}, "operand_bit_activity": {}}
    for comm in (0, 32, 64, 128, 192):
        out["active_compute_units"][str(256 - comm)] = run((256 - comm) * 32, comm, A, B)
    out["operand_bit_activity"]["N(0,1)/sqrt(K)"] = out["active_compute_units"]["256"]
    ones_a = torch.full((8192, k), 0x3F80, dtype=torch.int16, device="cuda")
    ones_b = torch.full((k, n), 0x3F80, dtype=torch.int16, device="cuda")
    out["operand_bit_activity"]["all 1.0"] = run(8192, 0, ones_a, ones_b)
    ones_a.zero_()
    ones_b.zero_()
    out["operand_bit_activity"]["all 0.0"] = run(8192, 0, ones_a, ones_b)
    del ones_a, ones_b
    # the governor's answer to a load that starts from idle: time per launch against the time since the first launch
    import time as _t
    torch.cuda.synchronize()
    _t.sleep(0.5)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(41)]
    evs[0].record(stream)
    for i in range(40):
        for _ in range(5):
            pk.pk_ag_gemm(1, 0, 8192, n, k, "bf16", A, B, None, None, None, 1, C, status)
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    t, ramp = 0.0, []
    for i in range(40):
        dt = evs[i].elapsed_time(evs[i + 1])
        t += dt
        if i in (0, 1, 2, 4, 7, 11, 15, 19, 24, 29, 34, 39):
            ramp.append([round(t, 1), round(dt / 5, 4)])
    out["ms_per_launch_against_ms_since_start_from_idle"] = ramp
    return out


def extras(pk, wl, torch, np, L):
    """Informational timings: bare GEMM, reduce and gather phases alone, live arrival."""
    c3, c4, rank = L["c3"], L["c4"], L["rank"]
    stream = L["stream"]
    out = {}

    def timeit(fn, n=10, w=3, st=None):
        st = st or stream
        for _ in range(w):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(st)
        for _ in range(n):
            fn()
        b.record(st)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    # bare GEMM of the cfg3 local shape with bf16 output (P = 1 all-gather GEMM): the "GEMM" column of the paper's Table 3
    m, n, k = c3.local_mnk
    Cg = torch.zeros((m, n), dtype=torch.int16, device="cuda")
    t_gemm = timeit(lambda: pk.pk_ag_gemm(1, 0, m, n, k, "bf16", L["A3"], L["B3"], None, None, None, 1, Cg, L["status"]))
    ep = [10 ** 6]

    def fused():
        ep[0] += 1
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                      L["flags_in"], L["flags_out"], ep[0], L["out3"], pk.PHASE_ALL, L["status"])
    t_fused = timeit(fused)
    out["table3_style"] = {"gemm_ms": round(t_gemm, 4), "gemm_rs_ms": round(t_fused, 4),
                           "comm_ratio": round((t_fused - t_gemm) / t_fused, 4)}
    # context only: the ROCm library GEMM (torch.matmul) on the same operands, i.e. the same data-dependent power draw
    Ab, Bb = L["A3"].view(torch.bfloat16), L["B3"].view(torch.bfloat16)
    Cl = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    t_lib = timeit(lambda: torch.matmul(Ab, Bb, out=Cl))
    out["table3_style"]["library_gemm_ms"] = round(t_lib, 4)
    out["table3_style"]["gemm_TFLOP/s"] = round(c3.flops / (t_gemm * 1e-3) / 1e12, 1)
    out["table3_style"]["library_gemm_TFLOP/s"] = round(c3.flops / (t_lib * 1e-3) / 1e12, 1)

    # the same bare GEMM on operands without bit activity (all 1.0): what the kernel's instruction schedule delivers when
    # data-dependent power does not hold the clock down
    ones_a = torch.full((m, k), 0x3F80, dtype=torch.int16, device="cuda")
    ones_b = torch.full((k, n), 0x3F80, dtype=torch.int16, device="cuda")
    t_ones = timeit(lambda: pk.pk_ag_gemm(1, 0, m, n, k, "bf16", ones_a, ones_b, None, None, None, 1, Cg, L["status"]))
    t_lib_ones = timeit(lambda: torch.matmul(ones_a.view(torch.bfloat16), ones_b.view(torch.bfloat16), out=Cl))
    out["table3_style"]["gemm_constant_operands_ms"] = round(t_ones, 4)
    out["table3_style"]["gemm_constant_operands_TFLOP/s"] = round(c3.flops / (t_ones * 1e-3) / 1e12, 1)
    out["table3_style"]["library_gemm_constant_operands_TFLOP/s"] = round(c3.flops / (t_lib_ones * 1e-3) / 1e12, 1)
    del ones_a, ones_b

    # gather phase alone: the emulated communicator moving the 7 peer chunks (read + write), by workgroup count
    staging = L["A4"].clone()
    counters = torch.zeros(pk.EMU_MAX_ORDER, dtype=torch.int32, device="cuda")
    order = L["i4"]["order"]
    moved = 2 * (c4.P - 1) * (c4.M // c4.P) * c4.K * 2
    out["gather_phase"] = {}
    for n_wg in (32, 256, 1024):
        def gather():
            counters.zero_()
            pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], L["chunk_flags"], 0x7FFFFFFF, order, 0,
                                     counters, n_wg=n_wg)
        t_g = timeit(gather)
        out["gather_phase"][f"{n_wg} workgroups"] = {"ms": round(t_g, 4), "GB/s": round(moved / (t_g * 1e-3) / 1e9, 1),
                                                     "frac_of_hbm_peak": round(moved / (t_g * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}

    def live(COMM):
        # live runs on a compute-unit partition (the paper's SM split): COMM compute units (COMM/8 per XCD) run the
        # emulated communicator on one stream, the op runs on the others through a second stream; flags start below the
        # epoch every iteration.  Feeder: 8 workgroups per communicator compute unit.
        h_comp, h_comm = pk.pk_partition_create(COMM)
        comp, side = torch.cuda.ExternalStream(h_comp), torch.cuda.ExternalStream(h_comm)
        flags_live = torch.zeros(c4.P, dtype=torch.int32, device="cuda")
        done = torch.cuda.Event()
        ep4 = [2 * 10 ** 6]
        torch.cuda.synchronize()

        def ag_live():
            ep4[0] += 1
            done.record(comp)
            side.wait_event(done)
            with torch.cuda.stream(side):
                counters.zero_()
            pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_live, ep4[0], order, 0, counters,
                                     stream=side, n_wg=8 * COMM)
            pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, flags_live, ep4[0], L["C4"],
                          L["status"], comm_cus=COMM, stream=comp)
            comp.wait_stream(side)
        t_live = timeit(ag_live, st=comp)
        t_pre224 = timeit(lambda: pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None,
                                                L["chunk_flags"], 1, L["C4"], L["status"], comm_cus=COMM, stream=comp), st=comp)

        def feeder_alone():
            with torch.cuda.stream(side):
                counters.zero_()
            pk.pk_emu_deliver_chunks(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_live, 1, order, 0, counters,
                                     stream=side, n_wg=8 * COMM)
        t_feed = timeit(feeder_alone, st=side)
        res = {}
        res["ag_gemm_live"] = {"ms_live_ring_arrival": round(t_live, 4), "ms_prelanded_224_cus": round(t_pre224, 4),
                               "ms_feeder_alone": round(t_feed, 4), "comm_cus": COMM,
                               "TFLOP/s_live": round(c4.flops / (t_live * 1e-3) / 1e12, 1)}

        # live reduce-scatter: the 7 peer slots arrive tile by tile through the emulated communicator
        flags_live3 = torch.zeros_like(L["flags_in"])
        stage3 = L["part"].clone()
        p3 = L["p3"]
        peers = [q for q in range(c3.P) if q != rank]
        ep3 = [3 * 10 ** 6]
        torch.cuda.synchronize()

        def rs_live():
            ep3[0] += 1
            done.record(comp)
            side.wait_event(done)
            pk.pk_emu_deliver_partials(c3.P, c3.M, c3.N, p3.tile_m, p3.tile_n, stage3, L["part"], flags_live3, ep3[0],
                                       peers, 0, stream=side, n_wg=8 * COMM)
            pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                          flags_live3, L["flags_out"], ep3[0], L["out3"], pk.PHASE_ALL, L["status"], comm_cus=COMM, stream=comp)
            comp.wait_stream(side)
        t_rs_live = timeit(rs_live, st=comp)
        ep3b = [4 * 10 ** 6]

        def rs_pre224():
            ep3b[0] += 1
            pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                          L["flags_in"], L["flags_out"], ep3b[0], L["out3"], pk.PHASE_ALL, L["status"], comm_cus=COMM, stream=comp)
        t_rs_pre224 = timeit(rs_pre224, st=comp)
        res["gemm_rs_live"] = {"ms_live_peer_partials": round(t_rs_live, 4), "ms_prelanded_224_cus": round(t_rs_pre224, 4),
                               "ms_prelanded_256_cus": out["table3_style"]["gemm_rs_ms"], "comm_cus": COMM}
        torch.cuda.synchronize()
        pk.pk_partition_destroy(h_comp, h_comm)
        return res

    # chunks moved by device-to-device copies + stream flag writes (no communicator workgroups), GEMM on all compute units
    side2 = torch.cuda.Stream()
    flags_dma = torch.zeros(c4.P, dtype=torch.int32, device="cuda")
    done2 = torch.cuda.Event()
    epd = [8 * 10 ** 6]

    def ag_live_dma():
        epd[0] += 1
        done2.record(stream)
        side2.wait_event(done2)
        pk.pk_emu_deliver_chunks_dma(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_dma, epd[0], order, stream=side2)
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, flags_dma, epd[0], L["C4"],
                      L["status"])
        stream.wait_stream(side2)
    t_dma = timeit(ag_live_dma)
    ring = list(order)
    order = ring[::-1]                      # adversarial: the chunk the schedule wants first arrives last
    t_dma_rev = timeit(ag_live_dma)
    order = ring
    t_dma_alone = timeit(lambda: pk.pk_emu_deliver_chunks_dma(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_dma, 1, order,
                                                               stream=stream))
    out["ag_gemm_live_copy_engine"] = {"ms_live_ring_arrival": round(t_dma, 4), "ms_live_reverse_arrival": round(t_dma_rev, 4),
                                       "ms_copies_alone": round(t_dma_alone, 4),
                                       "TFLOP/s_live": round(c4.flops / (t_dma * 1e-3) / 1e12, 1)}

    # all-gather along the last dimension of A (column chunks, strided copies) at the cfg4 shape
    def ag_k_pre():
        pk.pk_ag_gemm_k(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, L["chunk_flags"], 1, L["C4"],
                        L["status"])
    t_k_pre = timeit(ag_k_pre)

    def ag_k_live():
        epd[0] += 1
        done2.record(stream)
        side2.wait_event(done2)
        pk.pk_emu_deliver_kchunks_dma(c4.P, c4.M, c4.K, 2, staging, L["A4"], flags_dma, epd[0], order, stream=side2)
        pk.pk_ag_gemm_k(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, flags_dma, epd[0], L["C4"],
                        L["status"])
        stream.wait_stream(side2)
    t_k_live = timeit(ag_k_live)
    out["ag_gemm_last_dim_cfg4_shape"] = {"ms_prelanded": round(t_k_pre, 4), "ms_live_ring_arrival_strided_copies": round(t_k_live, 4),
                                          "TFLOP/s_prelanded": round(c4.flops / (t_k_pre * 1e-3) / 1e12, 1)}

    out.update(live(32))
    out["comm_cus_sweep"] = {}
    for cc in (16, 64):
        r = live(cc)
        out["comm_cus_sweep"][str(cc)] = {"ag_gemm_live_ms": r["ag_gemm_live"]["ms_live_ring_arrival"],
                                          "ag_feeder_alone_ms": r["ag_gemm_live"]["ms_feeder_alone"],
                                          "gemm_rs_live_ms": r["gemm_rs_live"]["ms_live_peer_partials"]}

    # GEMM + all-reduce at the cfg3 shape (one rank's share: the reduce phase also hands the reduced rows to the 7 peers)
    pa = pk.pk_gemm_ar_plan(c3.P, c3.M, c3.N, c3.K, c3.dtype)
    mp3 = c3.M // c3.P
    full = torch.zeros((c3.M, c3.N), dtype=torch.int16, device="cuda")
    bcast = torch.zeros((c3.P, mp3, c3.N), dtype=torch.int16, device="cuda")
    ar_in = torch.full((c3.P, pa.ar_flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    ar_in[rank].zero_()
    ar_out = torch.zeros_like(ar_in)
    epa = [5 * 10 ** 6]

    def ar(phases):
        def f():
            if phases & 1:
                epa[0] += 1
            pk.pk_gemm_ar(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, L["part"], L["outgoing"],
                          L["flags_in"], L["flags_out"], full, bcast, ar_in, ar_out, epa[0], phases, L["status"])
        return f
    t_ar = timeit(ar(pk.PHASE_ALL | pk.PHASE_WAIT))
    t_ar_red = timeit(ar(pk.PHASE_REDUCE))
    ar_red_bytes = c3.M * c3.N * 4 + c3.P * mp3 * c3.N * 2
    out["gemm_ar_cfg3_shape"] = {"ms": round(t_ar, 4), "TFLOP/s": round(c3.flops / (t_ar * 1e-3) / 1e12, 1),
                                 "reduce_and_hand_out_ms": round(t_ar_red, 4),
                                 "reduce_and_hand_out_GB/s": round(ar_red_bytes / (t_ar_red * 1e-3) / 1e9, 1)}

    # cfg5: fp8 e4m3 GEMM+RS (HBM-bound: 2.28 GB of mandatory traffic for 1.1e12 flop)
    c5 = wl.CONFIGS["cfg5"]
    i5 = wl.gemm_rs_inputs(c5.P, c5.M, c5.N, c5.K, c5.dtype, rank, seed=0, order=c5.order)
    p5 = pk.pk_gemm_rs_plan(c5.P, c5.M, c5.N, c5.K, c5.dtype)
    mp5 = c5.M // c5.P
    A5, B5 = torch.from_numpy(i5["A_local"]).cuda(), torch.from_numpy(i5["B_local"]).cuda()
    sa5 = torch.tensor([float(i5["scale_a"])], dtype=torch.float32, device="cuda")
    sb5 = torch.tensor([float(i5["scale_b"])], dtype=torch.float32, device="cuda")
    part5 = torch.from_numpy(i5["partials"]).cuda()
    outg5 = torch.zeros((c5.P, mp5, c5.N), dtype=torch.float32, device="cuda")
    out5 = torch.zeros((mp5, c5.N), dtype=torch.int16, device="cuda")
    fin5 = torch.full((c5.P, p5.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    fin5[rank].zero_()
    fout5 = torch.zeros_like(fin5)
    ep5 = [0]

    def rs5(phases):
        def f():
            if phases & 1:
                ep5[0] += 1
            pk.pk_gemm_rs(c5.P, rank, c5.M, c5.N, c5.K, c5.dtype, A5, B5, sa5, sb5, part5, outg5, fin5, fout5, ep5[0], out5,
                          phases, L["status"])
        return f
    t5 = timeit(rs5(pk.PHASE_ALL), n=5, w=2)
    t5g = timeit(rs5(pk.PHASE_GEMM), n=5, w=2)
    t5r = timeit(rs5(pk.PHASE_REDUCE), n=5, w=2)
    bytes5 = 2 * c5.M * (c5.K // c5.P) + 2 * c5.M * c5.N * 4 + mp5 * c5.N * 2
    red5 = c5.M * c5.N * 4 + mp5 * c5.N * 2
    out["cfg5_fp8_gemm_rs"] = {"ms": round(t5, 4), "TFLOP/s": round(c5.flops / (t5 * 1e-3) / 1e12, 1),
                               "GB/s_mandatory_traffic": round(bytes5 / (t5 * 1e-3) / 1e9, 1),
                               "frac_of_hbm_peak": round(bytes5 / (t5 * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                               "gemm_phase_ms": round(t5g, 4), "gemm_phase_TFLOP/s": round(c5.flops / (t5g * 1e-3) / 1e12, 1),
                               "reduce_phase_ms": round(t5r, 4), "reduce_phase_GB/s": round(red5 / (t5r * 1e-3) / 1e9, 1)}
    # the MLP block of the paper's section 4.1 with real data flow: AG + GEMM (cfg4) with SiLU fused into its epilogue writes
    # H (8192 x 3584 bf16), which is the local operand of GEMM + RS (cfg3)
    H = torch.zeros((c4.M, c4.N // c4.P), dtype=torch.int16, device="cuda")
    epm = [7 * 10 ** 6]

    def mlp():
        epm[0] += 1
        pk.pk_ag_gemm(c4.P, rank, c4.M, c4.N, c4.K, c4.dtype, L["A4"], L["B4"], None, None, L["chunk_flags"], 1, H,
                      L["status"], act="silu")
        pk.pk_gemm_rs(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, H, L["B3"], None, None, L["part"], L["outgoing"],
                      L["flags_in"], L["flags_out"], epm[0], L["out3"], pk.PHASE_ALL, L["status"])
    t_mlp = timeit(mlp)
    out["mlp_block_cfg4_silu_cfg3"] = {"ms": round(t_mlp, 4),
                                       "TFLOP/s": round((c3.flops + c4.flops) / (t_mlp * 1e-3) / 1e12, 1)}

    # GEMM + reduce-scatter along the last dimension at the cfg3 shape (shard 8192 x 1024 instead of 1024 x 8192)
    pc = pk.pk_gemm_rs_cols_plan(c3.P, c3.M, c3.N, c3.K, c3.dtype)
    part_c = L["part"].view(c3.P, c3.M, c3.N // c3.P)              # same bytes, slots reinterpreted as [P][M][N/P]
    outg_c = L["outgoing"].view(c3.P, c3.M, c3.N // c3.P)
    out_c = torch.zeros((c3.M, c3.N // c3.P), dtype=torch.int16, device="cuda")
    fin_c = torch.full((c3.P, pc.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    fin_c[rank].zero_()
    fout_c = torch.zeros_like(fin_c)
    epc = [9 * 10 ** 6]

    def rs_cols():
        epc[0] += 1
        pk.pk_gemm_rs_cols(c3.P, rank, c3.M, c3.N, c3.K, c3.dtype, L["A3"], L["B3"], None, None, part_c, outg_c, fin_c, fout_c,
                           epc[0], out_c, pk.PHASE_ALL, L["status"])
    t_cols = timeit(rs_cols)
    out["gemm_rs_last_dim_cfg3_shape"] = {"ms": round(t_cols, 4), "TFLOP/s": round(c3.flops / (t_cols * 1e-3) / 1e12, 1)}

    # the two small configurations are launch-latency bound: per-call time eager and as a HIP graph replay
    c1, c2 = wl.CONFIGS["cfg1"], wl.CONFIGS["cfg2"]
    i1 = wl.gemm_rs_inputs(c1.P, c1.M, c1.N, c1.K, c1.dtype, 0, seed=0)
    i2 = wl.ag_gemm_inputs(c2.P, c2.M, c2.N, c2.K, c2.dtype, 0, seed=0, order=c2.order)
    p1 = pk.pk_gemm_rs_plan(c1.P, c1.M, c1.N, c1.K, c1.dtype)
    A1, B1 = torch.from_numpy(i1["A_local"].view(np.int16)).cuda(), torch.from_numpy(i1["B_local"].view(np.int16)).cuda()
    part1 = torch.from_numpy(i1["partials"]).cuda()
    outg1 = torch.zeros_like(part1)
    fin1 = torch.full((c1.P, p1.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
    fin1[0].zero_()
    fout1 = torch.zeros_like(fin1)
    out1 = torch.zeros((c1.M // c1.P, c1.N), dtype=torch.int16, device="cuda")
    A2 = torch.from_numpy(np.concatenate(i2["chunks"], axis=0).view(np.int16)).cuda()
    B2 = torch.from_numpy(i2["B_local"].view(np.int16)).cuda()
    C2 = torch.zeros((c2.M, c2.N // c2.P), dtype=torch.int16, device="cuda")
    cf2 = torch.full((c2.P,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")

    def small(st=None):
        pk.pk_gemm_rs(c1.P, 0, c1.M, c1.N, c1.K, c1.dtype, A1, B1, None, None, part1, outg1, fin1, fout1, 1, out1,
                      pk.PHASE_ALL, L["status"], stream=st)
        pk.pk_ag_gemm(c2.P, 0, c2.M, c2.N, c2.K, c2.dtype, A2, B2, None, None, cf2, 1, C2, L["status"], stream=st)
    t_small = timeit(small, n=50, w=5)
    gs = torch.cuda.Stream()
    gs.wait_stream(stream)
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.stream(gs):
        small(gs)
        gs.synchronize()
        with torch.cuda.graph(gr, stream=gs):
            small(gs)
    torch.cuda.synchronize()
    t_graph = timeit(gr.replay, n=50, w=5)
    out["small_configs_cfg1_plus_cfg2"] = {"us_eager": round(t_small * 1e3, 1), "us_hip_graph_replay": round(t_graph * 1e3, 1),
                                           "kernels_per_call": 3}

    # the paper's own element size for communicated tiles (s = 2): bf16 partial slots halve scatter and reduce traffic
    out["bf16_partial_slots"] = {}
    for name, c, A, B, sa, sb, part32, fin, fout, o in (("cfg3", c3, L["A3"], L["B3"], None, None, L["part"], L["flags_in"],
                                                         L["flags_out"], L["out3"]),
                                                        ("cfg5", c5, A5, B5, sa5, sb5, part5, fin5, fout5, out5)):
        ep = [6 * 10 ** 6]
        outg32 = L["outgoing"] if name == "cfg3" else outg5
        pk.pk_gemm_rs(c.P, rank, c.M, c.N, c.K, c.dtype, A, B, sa, sb, part32, outg32, fin, fout, ep[0], o, pk.PHASE_ALL,
                      L["status"])
        torch.cuda.synchronize()
        ref_bits = o.clone()                                   # the fp32-slot result on the same inputs
        part16 = part32.to(torch.bfloat16).view(torch.int16)
        outg16 = torch.zeros(part16.shape, dtype=torch.int16, device="cuda")

        def rs16(phases):
            def f():
                if phases & 1:
                    ep[0] += 1
                pk.pk_gemm_rs(c.P, rank, c.M, c.N, c.K, c.dtype, A, B, sa, sb, part16, outg16, fin, fout, ep[0], o, phases,
                              L["status"], partial_dtype="bf16")
            return f
        t_all = timeit(rs16(pk.PHASE_ALL), n=10, w=3)
        t_g = timeit(rs16(pk.PHASE_GEMM), n=10, w=3)
        t_r = timeit(rs16(pk.PHASE_REDUCE), n=10, w=3)
        got = o.view(torch.bfloat16).float()
        ref = ref_bits.view(torch.bfloat16).float()
        out["bf16_partial_slots"][name] = {
            "ms": round(t_all, 4), "gemm_phase_ms": round(t_g, 4), "reduce_phase_ms": round(t_r, 4),
            "TFLOP/s": round(c.flops / (t_all * 1e-3) / 1e12, 1),
            "max_abs_diff_vs_fp32_slots_over_rms": round(((got - ref).abs().max() / ref.pow(2).mean().sqrt()).item(), 5)}
    # the paper's Table 3 (section 3.1.3) at its own sizes: M = N = 32768 per rank, local K from 512 to 8192, P = 8; bare
    # GEMM (bf16 output) against GEMM + reduce-scatter (fp32 slots, peers pre-landed); operands drawn on the device
    P8, MN = 8, 32768
    gen = torch.Generator(device="cuda")
    gen.manual_seed(251113940)
    mp8 = MN // P8
    part_t = torch.randn((P8, mp8, MN), generator=gen, device="cuda", dtype=torch.float32) * 0.01
    outg_t = torch.empty_like(part_t)
    out_t = torch.zeros((mp8, MN), dtype=torch.int16, device="cuda")
    C_t = torch.zeros((MN, MN), dtype=torch.int16, device="cuda")
    out["table3_paper_sizes"] = {}
    ept = [10 * 10 ** 6]
    for kl in (512, 1024, 2048, 4096, 8192):
        At = (torch.randn((MN, kl), generator=gen, device="cuda") / (P8 * kl) ** 0.5).to(torch.bfloat16).view(torch.int16)
        Bt = (torch.randn((kl, MN), generator=gen, device="cuda") / (P8 * kl) ** 0.5).to(torch.bfloat16).view(torch.int16)
        pt = pk.pk_gemm_rs_plan(P8, MN, MN, P8 * kl, "bf16")
        fin_t = torch.full((P8, pt.flags_per_slot), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
        fin_t[rank].zero_()
        fout_t = torch.zeros_like(fin_t)

        def rs_t(phases):
            def f():
                ept[0] += 1
                pk.pk_gemm_rs(P8, rank, MN, MN, P8 * kl, "bf16", At, Bt, None, None, part_t, outg_t, fin_t, fout_t, ept[0], out_t,
                              phases, L["status"])
            return f
        t_g = timeit(lambda: pk.pk_ag_gemm(1, 0, MN, MN, kl, "bf16", At, Bt, None, None, None, 1, C_t, L["status"]), n=5, w=3)
        t_s = timeit(rs_t(pk.PHASE_ALL), n=5, w=3)
        t_f = timeit(rs_t(pk.PHASE_ALL | pk.PHASE_OVERLAP), n=5, w=3)
        fl = 2.0 * MN * MN * kl
        out["table3_paper_sizes"][f"K={kl}"] = {"gemm_ms": round(t_g, 3), "gemm_rs_ms": round(t_f, 3),
                                                "comm_ratio": round((t_f - t_g) / t_f, 3),
                                                "gemm_rs_serial_reduce_ms": round(t_s, 3),
                                                "comm_ratio_serial_reduce": round((t_s - t_g) / t_s, 3),
                                                "gemm_TFLOP/s": round(fl / (t_g * 1e-3) / 1e12, 1),
                                                "gemm_rs_TFLOP/s": round(fl / (t_f * 1e-3) / 1e12, 1)}
        del At, Bt
    assert L["status"][0].item() == 0
    return out


if __name__ == "__main__":
    main()
