#!/usr/bin/env python3
"""Benchmark of the QUIK linear layer on one MI355X.

A step is one pass of the whole hot path (split + quantize, INT GEMM,
dequantization epilogue, fp16 outlier GEMM) over one synthetic batch, through the
C ABI (`quik_linear`, two kernel launches).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # dense int8 MFMA, MI355X data sheet (5.0 POP/s)
PEAK_FP6_TOPS = 10100.0      # dense FP6 / FP4 matrix rate, MI355X data sheet (10.1 PFLOP/s)
PEAK_SP24_TOPS = 10000.0     # 2:4-sparse int8 matrix rate counted in dense-equivalent operations: twice the
                             # dense int8 figure (the sparse instruction does a 64-column step in the time
                             # of a dense 32-column one)
PEAK_FP16_TFLOPS = 2500.0   # dense fp16 matrix rate, MI355X data sheet
PEAK_HBM_GBS = 8000.0
# profiles/gemm_stream_kernel_llama7b_up.md: (46193 KiB * 2.0 + 44032 KiB * 1.0) * 1024 for the persistent kernel;
# (47796 KiB * 2.0 + 44033 KiB * 1.0) * 1024 for the per-tile kernel (--gemm-path tiles)
TRAFFIC_BYTES = {"llama7b_up": int((46193 * 2.0 + 44032) * 1024)}
TRAFFIC_BYTES_TILES = {"llama7b_up": int((47796 * 2.0 + 44033) * 1024)}
# profiles/gemm_sp24_kernel_llama7b_up.md: the sparse GEMM, same factors
TRAFFIC_BYTES_SP24 = {"llama7b_up": int((47721 * 2.0 + 44034) * 1024)}


PREHEAT_MS = 150.0           # continuous load before any timing (the clocks need ~40-100 ms to settle)
MIN_EVENT_ITERS = 200        # launches per HIP-event timing of a single kernel
MIN_TIMED_MS = 200.0         # the --steps batch is repeated until this much has been timed


def _event_ms(fn, iters, torch):
    """Average duration of fn() in ms over `iters` back-to-back launches, measured with
    HIP events recorded on the stream the kernels are launched on (torch's current one)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def _preheat(fn, torch, ms=PREHEAT_MS):
    """Run fn() back to back for at least `ms` of GPU time, whatever --warmup says: after idle the
    chip runs short bursts up to 20 % slower than its sustained rate.  Returns the ms spent."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while True:
        for _ in range(50):
            fn()
        torch.cuda.synchronize()
        spent = (time.perf_counter() - t0) * 1e3
        if spent >= ms:
            return spent


def _kernel_ms(fn, torch, iters=MIN_EVENT_ITERS):
    """HIP-event time of one launch of fn at sustained clocks: a short pre-heat with the same launch,
    then the average over `iters` back-to-back launches."""
    _preheat(fn, torch, 30.0)
    return _event_ms(fn, iters, torch)


def cpu_baseline(inp, shp, budget_s=15.0):
    """The oracle as it stands, on this host's cores, on a bounded sample of token rows
    (tokens are independent, so a row sample is a faithful fraction of the workload)."""
    import numpy as np
    import oracle
    rows = min(64, shp.T)
    t0 = time.perf_counter()
    oracle.linear(inp.x[:rows], inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out)
    probe = time.perf_counter() - t0
    # the probe includes the per-call weight unpack; size the sample for ~budget_s
    rows = int(max(8, min(shp.T, rows * budget_s / max(probe, 1e-3))))
    t0 = time.perf_counter()
    oracle.linear(inp.x[:rows], inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out)
    dt = time.perf_counter() - t0
    tops = 2.0 * rows * shp.K * shp.N / dt / 1e12
    return {"value": tops, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {shp.T} token rows x all {shp.N} outputs, "
                      f"whole layer incl. weight unpack, {dt:.2f} s"}


def run_sweep(args, shp, torch, api, synth):
    """Layer time against token count or outlier count (the paper's appendix sweeps), with the
    FP16 GEMM of the same shape beside it.  One JSON object; not the headline metric."""
    import dataclasses
    dev = "cuda"
    rows = []
    if args.sweep == "tokens":
        points = [dataclasses.replace(shp, T=t) for t in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024,
                                                          2048, 4096, 8192)]
    else:
        points = [dataclasses.replace(shp, n_out=n) for n in (0, 64, 128, 256, 512, 1024)]
    for p in points:
        inp = synth.make_inputs(p)
        x = torch.from_numpy(inp.x).to(dev)
        idx = torch.from_numpy(inp.outlier_idx).to(dev) if p.n_out else None
        w_q = torch.from_numpy(inp.w_packed).to(dev)
        w_scale = torch.from_numpy(inp.w_scale).to(dev)
        w_out = torch.from_numpy(inp.w_out).to(dev) if p.n_out else None
        w_red = api.quik_weight_reduce(w_q, w_scale, p.K_b, p.bits)
        ws = torch.empty(api.quik_workspace_bytes(p.T, p.K, p.N, p.n_out, p.bits), dtype=torch.uint8,
                         device=dev)
        y = torch.empty((p.T, p.N), dtype=torch.float16, device=dev)
        step, _ = api.prepare_linear(x, idx, p.bits, w_q, w_scale, w_red, w_out, out=y, workspace=ws)
        for _ in range(args.warmup):
            step()
        ms = _event_ms(step, args.steps, torch)
        wf = (torch.randn((p.N, p.K), device=dev, dtype=torch.float32) * 0.02).to(torch.float16)
        for _ in range(5):
            torch.nn.functional.linear(x, wf)
        ms16 = _event_ms(lambda: torch.nn.functional.linear(x, wf), args.steps, torch)
        row = {"T": p.T, "n_out": p.n_out, "quik_ms": ms, "fp16_ms": ms16, "speedup": ms16 / ms,
               "tops": 2.0 * p.T * p.K * p.N / (ms * 1e-3) / 1e12}
        del wf
        if p.bits == 4 and p.weight_bits == 4 and p.K <= 16384:
            # the other two forms of the 4-bit layer on the same shape (the sparse one on the same
            # weights with two of every four base columns cleared)
            w6 = api.quik_weight_pack_fp6(w_q, p.K_b)
            step6, _ = api.prepare_linear_fp6(x, idx, w6, w_scale, w_red, w_out, out=y)
            for _ in range(max(5, args.warmup // 4)):
                step6()
            row["fp6_ms"] = _event_ms(step6, args.steps, torch)
            del w6, step6
            if p.K_b % 4 == 0:
                inp_s = synth.make_inputs(dataclasses.replace(p, sparse24=True))
                w_qs = torch.from_numpy(inp_s.w_packed).to(dev)
                w_red_s = api.quik_weight_reduce(w_qs, w_scale, p.K_b, 4)
                w24 = api.quik_weight_pack_sp24(w_qs, p.K_b)
                step24, _ = api.prepare_linear_sp24(x, idx, w24, w_scale, w_red_s, w_out, out=y)
                for _ in range(max(5, args.warmup // 4)):
                    step24()
                row["sp24_ms"] = _event_ms(step24, args.steps, torch)
                del w24, step24, w_qs, inp_s
        rows.append(row)
        del x, w_q, y, ws
    return {"sweep": args.sweep, "workload": f"{shp.name}: K={shp.K} N={shp.N} bits={shp.bits}",
            "steps": args.steps, "rows": rows}


def run_only(args, api, torch, shp, x, idx, w_q, w_scale, w_red, w_out, y, ws, step):
    """--only: `--steps` launches of one kernel on the workload's buffers, for counter runs."""
    import dataclasses
    from paper_2310_09259_amd import synth
    T, K, N, K_b, n_out, bits = shp.T, shp.K, shp.N, shp.K_b, shp.n_out, shp.bits
    xo = lambda q: q[3] if n_out else None
    if args.only == "layer":
        fn = step
    elif args.only == "quantize":
        fn = api.prepare_quantize(x, idx, bits, api.quik_quantize(x, idx, bits))
    elif args.only == "gemm":
        q = api.quik_quantize(x, idx, bits)
        fn = api.prepare_gemm_dequant(q[0], q[1], q[2], xo(q), K_b, bits, w_q, w_scale, w_red, w_out, None, y, q[4])
    elif args.only == "gemm_fp6":
        w6 = api.quik_weight_pack_fp6(w_q, K_b)
        q = api.quik_quantize_fp6(x, idx)
        fn = api.prepare_gemm_dequant_fp6(q[0], q[1], q[2], xo(q), K_b, w6, w_scale, w_red, w_out, None, y)
    elif args.only == "gemm_sp24":
        inp_s = synth.make_inputs(dataclasses.replace(shp, sparse24=True))
        w_qs = torch.from_numpy(inp_s.w_packed).to("cuda")
        w_red_s = api.quik_weight_reduce(w_qs, w_scale, K_b, 4)
        w24 = api.quik_weight_pack_sp24(w_qs, K_b)
        q = api.quik_quantize_sp24(x, idx)
        fn = api.prepare_gemm_dequant_sp24(q[0], q[1], q[2], xo(q), K_b, w24, w_scale, w_red_s, w_out, None, y)
    else:                                       # a kernel of known traffic, to scale FETCH_SIZE / WRITE_SIZE
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        fn = lambda: api.quik_debug_copy_probe(src, dst)
    for _ in range(args.warmup):
        fn()
    torch.cuda.synchronize()
    ms = _event_ms(fn, args.steps, torch)
    print(json.dumps({"only": args.only, "workload": shp.name, "launches": args.steps, "ms_per_launch": ms}))


def run_mix_probe(api, torch):
    """What each kind of instruction of the 4-bit GEMM's K loop costs the matrix pipe: the probe's rate for
    the matrix instruction alone and with vector operations, LDS reads, global -> LDS copies and barriers
    added at the K loop's counts, and the clock the chip held under each load."""
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    src = torch.randint(0, 255, (32 << 20,), dtype=torch.uint8, device=dev)
    clocks = torch.zeros(2, dtype=torch.int64, device=dev)
    iters = 4000
    names = {1: "changing random operands", 32: "as widened nibbles (4 varying bits per byte)",
             64: "on the 16x16x64 instruction (two per 32x32x32-equivalent, 8-byte LDS reads)", 2: "4 vector ops per MFMA",
             4: "5 LDS reads per 12 MFMAs", 8: "2 copies per 12 MFMAs", 16: "barrier per 48 MFMAs"}
    rows = []
    base = None
    _preheat(lambda: api.quik_debug_mix_probe(0, cus, iters, sink), torch)
    for mix in (0, 1, 3, 5, 9, 17, 7, 11, 13, 15, 31, 33, 35, 37, 41, 47, 63, 97, 127):
        call = lambda: api.quik_debug_mix_probe(mix, cus, iters, sink, src if mix & 8 else None, clocks)
        ops = call()
        ms = _kernel_ms(call, torch, 30)
        torch.cuda.synchronize()
        ck = clocks.cpu().numpy()
        tops = ops / (ms * 1e-3) / 1e12
        if base is None:
            base = tops
        rows.append({"mix": mix, "what": "MFMA alone, constant operands (small values)" if mix == 0 else
                     " + ".join(n for b, n in names.items() if mix & b),
                     "TOPS": tops, "frac_of_5_POPS": tops / PEAK_INT8_TOPS, "time_vs_first_row": base / tops,
                     "ns_per_mfma_per_simd": ms * 1e6 / (iters * 12 * 2),
                     # the shader clock held during the loop of wave 0 of workgroup 0: ticks of s_memtime per tick of
                     # the 100 MHz s_memrealtime over the same interval
                     "clock_MHz": 100.0 * float(ck[0]) / float(ck[1]) if ck[1] else None})
    print(json.dumps({"probe": "quik_debug_mix_probe", "workgroups": cus, "waves_per_workgroup": 8,
                      "mfma_per_iteration": 12, "iterations": iters, "rows": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The GPU's clocks take some tens of milliseconds of continuous load to reach their sustained
    # state (the first ~40 ms run up to 20 % slower), so the untimed warm-up is ~100 ms of steps.
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--workload", default="llama7b_up")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp16", action="store_true")
    ap.add_argument("--no-ablation", action="store_true",
                    help="skip the fusion-ablation timings (keeps a kernel trace down to the two "
                         "kernels of the layer and the FP16 comparator)")
    ap.add_argument("--graph", action="store_true",
                    help="replay a captured HIP graph holding one step instead of launching every "
                         "step through the binding (measured: no faster here, direct launches "
                         "already keep the queue full)")
    ap.add_argument("--sweep", choices=["tokens", "outliers"], default=None,
                    help="instead of the headline line, time the layer over a sweep of token counts "
                         "(1..8192) or outlier counts (0..1024) on the workload's K and N")
    ap.add_argument("--no-fp6", action="store_true",
                    help="skip the timing of the FP6-matrix-pipe form of the 4-bit layer")
    ap.add_argument("--no-sp24", action="store_true",
                    help="skip the timing of the 2:4-sparse form of the 4-bit layer")
    ap.add_argument("--only", choices=["layer", "gemm", "quantize", "gemm_fp6", "gemm_sp24", "copy"], default=None,
                    help="launch just this kernel (or the two of the layer) --steps times after --warmup "
                         "launches and exit: a short command line for rocprofv3 counter runs")
    ap.add_argument("--gemm-path", choices=["auto", "persistent", "tiles"], default="auto",
                    help="4-bit GEMM kernel family: the library's own choice (default), the persistent kernel "
                         "wherever it can run, or the per-tile kernels only (for profiles of either one)")
    ap.add_argument("--mix-probe", action="store_true",
                    help="instead of the layer: the K loop's instruction mix around the int8 matrix instruction, "
                         "one ingredient at a time (quik_debug_mix_probe); one JSON line with a row per mix")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain device-to-device copy of 256 MiB (a kernel of known "
                         "traffic, to scale the FETCH_SIZE / WRITE_SIZE counters of a --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU only: the layer shards over tokens with no "
              "communication, so runs on several GPUs are not part of this build (use --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2310_09259_amd import api, synth

    api.load()                      # fails loudly if the HIP library is missing
    api.quik_debug_set_gemm_path({"auto": 0, "persistent": 1, "tiles": 2}[args.gemm_path])
    if args.mix_probe:
        run_mix_probe(api, torch)
        return
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    shp = synth.CONFIGS[args.workload]
    if args.sweep:
        print(json.dumps(run_sweep(args, shp, torch, api, synth)))
        return
    inp = synth.make_inputs(shp)
    dev = "cuda"
    x = torch.from_numpy(inp.x).to(dev)
    idx = torch.from_numpy(inp.outlier_idx).to(dev) if shp.n_out else None
    w_q = torch.from_numpy(inp.w_packed).to(dev)
    w_scale = torch.from_numpy(inp.w_scale).to(dev)
    w_out = torch.from_numpy(inp.w_out).to(dev) if shp.n_out else None
    w_red = api.quik_weight_reduce(w_q, w_scale, shp.K_b, shp.weight_bits)
    T, K, N, K_b, n_out, bits = shp.T, shp.K, shp.N, shp.K_b, shp.n_out, shp.bits
    mixed = shp.weight_bits != bits        # 4-bit weights under 8-bit activations
    ws = torch.empty(api.quik_workspace_bytes(T, K, N, n_out, bits), dtype=torch.uint8, device=dev)
    y = torch.empty((T, N), dtype=torch.float16, device=dev)

    # one C-ABI call per step; its arguments are marshalled once (host time per call ~1 us).  A
    # prepared call is bound to the stream it was made on, so graph capture uses the plain call.
    if mixed:
        step, _ = api.prepare_linear_w4a8(x, idx, w_q, w_scale, w_red, w_out, out=y, workspace=ws)
    elif args.graph:
        def step():
            api.quik_linear(x, idx, bits, w_q, w_scale, w_red, w_out, out=y, workspace=ws)
    else:
        step, _ = api.prepare_linear(x, idx, bits, w_q, w_scale, w_red, w_out, out=y, workspace=ws)

    # --graph: the timed region replays a HIP graph that holds one step (both launches, captured
    # from the same C-ABI call on the capture stream).
    graph = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    run = graph.replay if graph is not None else step
    if args.only:
        # a short, single-kernel command line for counter runs (rocprofv3 --pmc): `--steps` launches of
        # one kernel, nothing else
        run_only(args, api, torch, shp, x, idx, w_q, w_scale, w_red, w_out, y, ws, step)
        return
    preheat_ms = _preheat(run, torch)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    # EXACTLY --steps steps per timed batch, bracketed by synchronizations; the batch is repeated until
    # MIN_TIMED_MS have been timed and the median batch is reported
    batches = []
    while True:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        batches.append((time.perf_counter() - t0) * 1e3)
        if sum(batches) >= MIN_TIMED_MS and len(batches) >= 3:
            break
    ms_step = float(np.median(batches)) / args.steps

    # per-kernel durations (HIP events on the launch stream), same buffers
    q_out = api.quik_quantize(x, idx, bits)
    xq, scale, zero, x_out, side = q_out
    it = max(MIN_EVENT_ITERS, args.steps // 2)
    quant_call = api.prepare_quantize(x, idx, bits, q_out)
    if mixed:
        def gemm_call():
            api.quik_gemm_dequant_w4a8(xq, scale, zero, x_out if n_out else None, K_b, w_q, w_scale, w_red,
                                       w_out, out=y)
    else:
        gemm_call = api.prepare_gemm_dequant(xq, scale, zero, x_out if n_out else None, K_b, bits, w_q,
                                             w_scale, w_red, w_out, None, y, side)
    ms_quant = _kernel_ms(quant_call, torch, it)
    ms_gemm = _kernel_ms(gemm_call, torch, it)
    # The same GEMM launch on operands without entropy (every packed byte 0x88 = all codes zero in the
    # activations' and the weights' nibble order alike): same instruction stream, same bytes moved.  The chip
    # holds a higher clock when the operand bits do not toggle; the difference to ms_gemm is what the
    # benchmark's uniformly random codes cost in clock, not in work.
    ms_gemm_flat = None
    if not mixed:
        xq_flat, wq_flat = torch.full_like(xq, 0x88), torch.full_like(w_q, 0x88)
        flat_call = api.prepare_gemm_dequant(xq_flat, scale, zero, x_out if n_out else None, K_b, bits, wq_flat,
                                             w_scale, w_red, w_out, None, y, side)
        ms_gemm_flat = _kernel_ms(flat_call, torch, it)
        del xq_flat, wq_flat, flat_call
    ms_layer_ev = _kernel_ms(step, torch, it)

    # the quantization kernel on inputs that are NOT cache-resident: a rotation of distinct input and
    # output buffer sets larger than the 256 MB last-level cache (the figure above re-reads one 17 MB
    # input, which stays in that cache)
    quant_bytes = T * (2 * K + K_b * bits // 8 + 2 * n_out + 8 + (4 if bits == 4 else 0))
    n_rot = max(32, int(2 * (256 << 20) / quant_bytes) + 1)
    rot_x = [x.clone() for _ in range(n_rot)]
    rot_out = [tuple(torch.empty_like(t) for t in q_out) for _ in range(n_rot)]
    rot_calls = [api.prepare_quantize(rx, idx, bits, ro) for rx, ro in zip(rot_x, rot_out)]

    def quant_rotation():
        for c in rot_calls:
            c()
    _preheat(quant_rotation, torch, 30.0)
    ms_quant_cold = _event_ms(quant_rotation, max(2, MIN_EVENT_ITERS // n_rot), torch) / n_rot
    del rot_x, rot_out, rot_calls

    # what the chip sustains: the int8 matrix instruction alone, and a plain streaming copy
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_ops = api.quik_debug_mfma_probe(2048, 2000, sink)
    ms_probe = _kernel_ms(lambda: api.quik_debug_mfma_probe(2048, 2000, sink), torch, 20)
    measured_mfma_tops = probe_ops / (ms_probe * 1e-3) / 1e12
    # the same instruction on operands of pseudo-random bytes (the chip lowers its clock under them), and with
    # the K loop's other instructions beside it (vector operations, LDS reads, copies, barriers; no dependences)
    cus_ = torch.cuda.get_device_properties(0).multi_processor_count
    mix_src = torch.randint(0, 255, (32 << 20,), dtype=torch.uint8, device=dev)
    mix_tops = {}
    for mix in (1, 31, 33, 63, 97, 127):
        mix_ops = api.quik_debug_mix_probe(mix, cus_, 2000, sink, mix_src if mix & 8 else None)
        ms_mix = _kernel_ms(lambda: api.quik_debug_mix_probe(mix, cus_, 2000, sink, mix_src if mix & 8 else None), torch, 20)
        mix_tops[mix] = mix_ops / (ms_mix * 1e-3) / 1e12
    del mix_src
    src = torch.empty(512 << 20, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    ms_copy = _kernel_ms(lambda: api.quik_debug_copy_probe(src, dst), torch, 20)
    measured_hbm_gbs = 2.0 * src.numel() / (ms_copy * 1e-3) / 1e9
    del src, dst

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # fusion ablation (Section 3.4, kernel versions 1-3), same buffers
    ws_abl = torch.empty(api.quik_ablation_workspace_bytes(T, K, N, n_out, bits), dtype=torch.uint8,
                         device=dev)
    ablation = {}
    no_ablation = args.no_ablation or mixed          # the unfused variants exist for equal widths only
    for version in (() if no_ablation else (1, 2, 3)):
        fn = lambda v=version: api.quik_linear_ablation(v, x, idx, bits, w_q, w_scale, w_red, w_out,
                                                        out=y, workspace=ws_abl)
        ablation[f"v{version}"] = _kernel_ms(fn, torch, it)
    del ws_abl

    # the same 4-bit layer with the integer product on the FP6 matrix pipe (exact; reported beside the
    # headline, which stays on the int8-MFMA path the benchmark spec names)
    fp6 = None
    if bits == 4 and not mixed and K <= 16384 and not args.no_fp6:
        w6 = api.quik_weight_pack_fp6(w_q, K_b)
        ws6 = torch.empty(api.quik_workspace_bytes_fp6(T, K, N, n_out), dtype=torch.uint8, device=dev)
        step6, _ = api.prepare_linear_fp6(x, idx, w6, w_scale, w_red, w_out, out=y, workspace=ws6)
        q6 = api.quik_quantize_fp6(x, idx)
        gemm6 = api.prepare_gemm_dequant_fp6(q6[0], q6[1], q6[2], q6[3] if n_out else None, K_b, w6, w_scale,
                                             w_red, w_out, None, y)
        quant6 = api.prepare_quantize_fp6(x, idx, q6)
        ms6_layer = _kernel_ms(step6, torch, it)
        ms6_gemm = _kernel_ms(gemm6, torch, it)
        ms6_quant = _kernel_ms(quant6, torch, it)
        fp6 = {"layer_ms": ms6_layer, "layer_TOPS": 2.0 * T * K * N / (ms6_layer * 1e-3) / 1e12,
               "kernels_ms": {"quik_quantize_fp6": ms6_quant, "quik_gemm_dequant_fp6": ms6_gemm},
               "roofline": {"bound": "mfma", "kernel": "gemm_fp6_kernel", "peak": PEAK_FP6_TOPS, "unit": "TOP/s",
                            "achieved": 2.0 * T * K_b * N / (ms6_gemm * 1e-3) / 1e12,
                            "frac": 2.0 * T * K_b * N / (ms6_gemm * 1e-3) / 1e12 / PEAK_FP6_TOPS},
               "operand_bytes_per_element": 0.75}
        del w6, ws6, q6

    # the 4-bit layer with 2:4-sparse weights on the sparse int8 matrix instruction: same shape, same
    # activations, the synthetic weights with two of every four base columns cleared (reported beside
    # the headline; rates count the dense-equivalent operations 2 T K N)
    sp24 = None
    if bits == 4 and not mixed and K <= 16384 and K_b % 4 == 0 and not args.no_sp24:
        import dataclasses
        inp_s = synth.make_inputs(dataclasses.replace(shp, sparse24=True))
        w_qs = torch.from_numpy(inp_s.w_packed).to(dev)
        w_red_s = api.quik_weight_reduce(w_qs, w_scale, K_b, 4)
        w24 = api.quik_weight_pack_sp24(w_qs, K_b)
        ws24 = torch.empty(api.quik_workspace_bytes_sp24(T, K, N, n_out), dtype=torch.uint8, device=dev)
        step24, _ = api.prepare_linear_sp24(x, idx, w24, w_scale, w_red_s, w_out, out=y, workspace=ws24)
        q24 = api.quik_quantize_sp24(x, idx)
        gemm24 = api.prepare_gemm_dequant_sp24(q24[0], q24[1], q24[2], q24[3] if n_out else None, K_b, w24,
                                               w_scale, w_red_s, w_out, None, y)
        quant24 = api.prepare_quantize_sp24(x, idx, q24)
        ms24_layer = _kernel_ms(step24, torch, it)
        ms24_gemm = _kernel_ms(gemm24, torch, it)
        ms24_quant = _kernel_ms(quant24, torch, it)
        sp24 = {"layer_ms": ms24_layer, "layer_TOPS_dense_equivalent": 2.0 * T * K * N / (ms24_layer * 1e-3) / 1e12,
                "kernels_ms": {"quik_quantize_sp24": ms24_quant, "quik_gemm_dequant_sp24": ms24_gemm},
                "roofline": {"bound": "mfma", "kernel": "gemm_sp24_kernel", "peak": PEAK_SP24_TOPS,
                             "unit": "TOP/s (dense-equivalent)",
                             "achieved": 2.0 * T * K_b * N / (ms24_gemm * 1e-3) / 1e12,
                             "frac": 2.0 * T * K_b * N / (ms24_gemm * 1e-3) / 1e12 / PEAK_SP24_TOPS,
                             "traffic": TRAFFIC_BYTES_SP24.get(args.workload)},
                "weight_bytes_per_element": 0.5, "activation_bytes_per_element": 0.5}
        del w24, ws24, q24, w_qs, inp_s

    ms_fp16 = ms_lib_int8 = None
    if not args.no_fp16:
        wf = (torch.randn((N, K), device=dev, dtype=torch.float32) * 0.02).to(torch.float16)
        ms_fp16 = _kernel_ms(lambda: torch.nn.functional.linear(x, wf), torch, it)
        del wf
        # context for the roofline fraction: the vendor library's plain int8 GEMM (operands already one
        # byte per value, no widening, no epilogue, no outlier product) on the integer part's shape
        try:
            ai = torch.randint(-8, 8, (T, K_b), dtype=torch.int8, device=dev)
            wi = torch.randint(-8, 8, (N, K_b), dtype=torch.int8, device=dev)
            ms_lib_int8 = _kernel_ms(lambda: torch._int_mm(ai, wi.t()), torch, it)
            del ai, wi
        except Exception:                                    # shapes the library call does not take
            ms_lib_int8 = None

    ops_layer = 2.0 * T * K * N
    ops_int = 2.0 * T * K_b * N
    # which kernel family the library picks for this shape (host logic of the library, asked through the ABI)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    plan = api.quik_debug_gemm_plan(T, N, K_b, cus) if (bits == 4 and not mixed) else None
    persistent = plan is not None and args.gemm_path != "tiles" and (plan[0] == 1 or args.gemm_path == "persistent")
    # per-tile family: gemm_tiles16_kernel runs the 256 x 128 tiles of equal operand widths, gemm_kernel /
    # gemm_skinny the other tiles (the dispatch in quik_gemm.hip decides)
    gemm_kernel_name = "gemm_stream_kernel" if persistent else "gemm_kernel|gemm_tiles16_kernel"
    tops = ops_layer / (ms_step * 1e-3) / 1e12
    gemm_tops = ops_int / (ms_gemm * 1e-3) / 1e12
    out = {
        "metric": "QUIK linear TOPS (whole layer: quantize + INT4 GEMM + dequant + fp16 outliers)",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "preheat_ms": preheat_ms, "timed_batches": len(batches),
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": (f"int{shp.weight_bits} weights x int{bits} activations" if mixed else f"int{bits} operands") +
                 " on int8 MFMA, int32 accumulate, fp16 outliers",
        "data": "synthetic",
        "config": {"workload": f"{shp.name}: T={T} K={K} N={N} n_out={n_out} bits={bits}" + (f" w_bits={shp.weight_bits}" if mixed else ""),
                   "launches_per_step": 2, "hip_graph_replay": graph is not None},
        "frac_int8_mfma_peak_layer": tops / PEAK_INT8_TOPS,
        "speedup_vs_fp16_gemm": (ms_fp16 / ms_step) if ms_fp16 else None,
        "fp16_gemm_ms": ms_fp16,
        "library_int8_gemm": None if ms_lib_int8 is None else {
            "ms": ms_lib_int8, "frac_int8_mfma_peak": ops_int / (ms_lib_int8 * 1e-3) / 1e12 / PEAK_INT8_TOPS,
            "what": "torch._int_mm (hipBLASLt) on [T, K_b] x [K_b, N] int8: context, not part of the path"},
        "kernels_ms": {"quik_quantize": ms_quant, "quik_gemm_dequant": ms_gemm,
                       "quik_linear_events": ms_layer_ev},
        "fusion_ablation_ms": None if no_ablation else {
            "v1_unfused_quant_unfused_dequant": ablation["v1"],
            "v2_fused_quant_unfused_dequant": ablation["v2"],
            "v3_fused_quant_fused_dequant": ablation["v3"]},
        "quantize_hbm": {"algorithmic_bytes": quant_bytes, "peak_GBs": PEAK_HBM_GBS,
                         "warm": {"ms": ms_quant, "achieved_GBs": quant_bytes / (ms_quant * 1e-3) / 1e9,
                                  "frac": quant_bytes / (ms_quant * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                  "what": "one input re-read: resident in the 256 MB last-level cache"},
                         "cold": {"ms": ms_quant_cold, "achieved_GBs": quant_bytes / (ms_quant_cold * 1e-3) / 1e9,
                                  "frac": quant_bytes / (ms_quant_cold * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                  "frac_of_measured_copy": quant_bytes / (ms_quant_cold * 1e-3) / 1e9 / measured_hbm_gbs,
                                  "what": f"rotation of {n_rot} distinct input/output sets "
                                          f"({n_rot * quant_bytes / 2**20:.0f} MiB): served by HBM"}},
        "measured_peaks": {"int8_mfma_TOPS": measured_mfma_tops,
                           "int8_mfma_TOPS_random_operands": mix_tops[1],
                           "int8_mfma_TOPS_k_loop_mix": mix_tops[31],
                           "int8_mfma_TOPS_nibble_operands": mix_tops[33],
                           "int8_mfma_TOPS_k_loop_mix_nibble_operands": mix_tops[63],
                           "int8_mfma_16x16x64_TOPS_nibble_operands": mix_tops[97],
                           "int8_mfma_16x16x64_TOPS_k_loop_mix_nibble_operands": mix_tops[127],
                           "copy_GBs": measured_hbm_gbs,
                           "what": "quik_debug_mfma_probe (independent 32x32x32 int8 matrix instructions on "
                                   "register-resident operands of small values), quik_debug_mix_probe 1 (the same on "
                                   "operands of pseudo-random bytes) and 31 (with the vector, LDS, copy and barrier "
                                   "instructions of the GEMM's K loop beside them, no dependences), 33 and 63 (as 1 and 31 "
                                   "on operand bytes of the kind the GEMM's nibble widening makes -- the ceiling for its own operands), 97 and 127 "
                                   "(as 33 and 63 on the 16 x 16 x 64 instruction of the persistent kernel), "
                                   "quik_debug_copy_probe (512 MiB streaming copy, read + write bytes)"},
        "roofline": {"bound": "mfma", "kernel": gemm_kernel_name + " (INT GEMM + dequant + outlier GEMM)",
                     "achieved": gemm_tops, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": gemm_tops / PEAK_INT8_TOPS,
                     "frac_of_measured_mfma_peak": gemm_tops / measured_mfma_tops,
                     "frac_of_measured_mfma_peak_random_operands": gemm_tops / mix_tops[1],
                     "frac_of_measured_k_loop_mix": gemm_tops / mix_tops[31],
                     "frac_of_measured_k_loop_mix_nibble_operands": gemm_tops / mix_tops[63],
                     # the persistent kernel's own instruction shape (the per-tile 32 x 32 forms: the row above)
                     "frac_of_measured_k_loop_mix_16x16x64": gemm_tops / mix_tops[127],
                     "same_launch_on_constant_operands": None if ms_gemm_flat is None else {
                         "ms": ms_gemm_flat, "frac": ops_int / (ms_gemm_flat * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                         "what": "every packed operand byte 0x88 (all codes zero): the clock the chip holds depends "
                                 "on how much the operand bits toggle"},
                     # the kernel's two contractions against their own peaks: time at 100 % of the int8 rate for
                     # the integer part plus time at 100 % of the fp16 rate for the outlier part, over the time taken
                     "frac_roof_int8_plus_fp16": (ops_int / (PEAK_INT8_TOPS * 1e12) + 2.0 * T * n_out * N / (PEAK_FP16_TFLOPS * 1e12))
                                                 / (ms_gemm * 1e-3),
                     # HBM-side bytes per launch from rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0
                     # (factors from a 256 MiB copy; see profiles/), measured for the default
                     # workload only
                     "traffic": (TRAFFIC_BYTES if persistent else TRAFFIC_BYTES_TILES).get(args.workload),
                     "algorithmic_ops_per_launch": ops_int},
    }
    if fp6 is not None:
        out["fp6_path"] = fp6
    if sp24 is not None:
        out["sp24_path"] = sp24
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, shp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
