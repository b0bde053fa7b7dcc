#!/usr/bin/env python3
"""Benchmark of the ChunkFT hot path on one MI355X.

Workload: configuration [1] of the task's list -- Llama-3-8B up_proj shape (W 14336 x 4096
bf16, T = 1024 tokens), one chunk of 32 Mi contiguous elements at a seeded
mid-row offset, synthetic Gaussian inputs already resident in HBM.

One step = one pass of every stage of the path over that batch:
  plan      chunkft_plan_cycle on the layer (host, integer)
  wgrad     chunkft_chunk_wgrad            -> fp32 g[chunk]
  adamw     chunkft_adamw_chunk            g -> master, m, v, bf16 W   (state set A)
  fused     chunkft_wgrad_adamw_fused      same update, g never stored  (state set B)

`value` is the chunk-wgrad rate 2*T*E / t(wgrad call) in TFLOP/s; the AdamW
GB/s (30 B/element) and the fused call are reported beside it.  Kernel times
are HIP-event brackets on the stream the kernels run on, taken inside the
timed region.  The CPU baseline is the fp64 oracle on the host cores.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0        # HBM3E

# HBM bytes per launch at this workload from rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE,
# each scaled by what the counter reads for the plain copy of --copy-probe: x2.000 and x1.000);
# the summary of those runs is profiles/bench_llama8b_upproj_hbm_traffic.txt.
MEASURED_TRAFFIC = {"wgrad": 237.8e6, "adamw": 1006.7e6, "fused": 1048.8e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-steps", type=int, default=100,
                    help="untimed steps before the warm-up steps (about 45 ms), so that the "
                         "device's clock management has settled under the load (0: none)")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the plain and the fused call at longer token counts (the same layer shape, "
                         "T = 4096 and 8192) and on the lm_head shape of configs[4] per chunk size; "
                         "reported under \"sweep\"")
    ap.add_argument("--stream-state", action="store_true",
                    help="also time the rotating schedule with the chunk state kept in pinned host memory "
                         "(three 32Mi-element chunks, interval 4, prefetch of the next chunk and offload of "
                         "the previous one beside the kernels); reported under \"streamed_state\"")
    ap.add_argument("--plan-sweep", action="store_true",
                    help="also run the cycle planner over the whole Llama-3-8B tensor list for several chunk "
                         "counts and report the byte imbalance and the memory jitter it implies, beside a "
                         "layer-wise partition (host only); reported under \"plan_sweep\"")
    ap.add_argument("--block-cycle", action="store_true",
                    help="also run one cycle over a whole Llama-3-8B transformer block (configs[2]: q, k, v, o, "
                         "gate, up, down and two norm vectors, T = 1024) with the planner's chunks for a 256 MiB "
                         "budget: one fused call per segment, timed per chunk; reported under \"block_cycle\"")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the \"per_config\" block (every other configuration of the task's list timed on "
                         "device-generated operands of its shapes, a few milliseconds each)")
    ap.add_argument("--timeline", nargs="?", const="wgrad", choices=("wgrad", "fused"),
                    help="instead of the benchmark: run the plain gradient (or, with `fused`, the fused call) of the workload through "
                         "libchunkft_timeline.so (the library built with the MFMA kernel's time stamps) and print "
                         "where each workgroup's time goes: start, first fragments in registers, end of loop, "
                         "end of epilogue, per compute unit")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region, run a plain device copy of known size (256 MiB read, "
                         "256 MiB written, three times): the calibration point for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no collective); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_21177_amd import binding as B
    from paper_2605_21177_amd import workloads as WL

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    case, begin, end = WL.config2()
    E = end - begin
    T = case.T
    X = case.X.to(dev)
    dY = case.dY.to(dev)
    layer = B.make_layer(B.LINEAR, X, dY, case.out, case.n_in)
    S = B.chunkft_split_k(layer, begin, end)
    ws_bytes = B.chunkft_workspace_bytes(layer, begin, end)
    ws = torch.empty(max(ws_bytes // 4, 1), dtype=torch.float32, device=dev) if ws_bytes else None
    tensors = [(case.out, case.n_in, case.dtype, case.kind)]
    budget = 64 << 20

    W = case.W0.reshape(-1).clone().to(dev)
    # chunk-local arrays in the layout the header recommends: the 128-byte phase of the tensor's rows
    g = B.chunk_array(E, begin, dev)

    def fresh_state(aligned=True):
        if not aligned:
            master = W[begin:end].float()
            return master, torch.zeros_like(master), torch.zeros_like(master)
        master, m, v = B.chunk_state(E, begin, dev)
        master.copy_(W[begin:end])
        m.zero_()
        v.zero_()
        return master, m, v

    stA = fresh_state()
    stB = fresh_state()
    Wa_slice = W.clone()[begin:end]
    Wb = W.clone()
    hp = dict(WL.HPARAMS)

    names = ("wgrad", "adamw", "fused")
    ev = {n: [] for n in names}

    def step(i, record):
        B.chunkft_plan_cycle(tensors, budget)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if record else None
        h = B.hparams(step=i + 1, **hp)
        if record: marks[0].record()
        B.chunkft_chunk_wgrad(layer, begin, end, g, ws=ws)
        if record: marks[1].record()
        B.chunkft_adamw_chunk(g, stA[0], stA[1], stA[2], Wa_slice, E, h)
        if record: marks[2].record()
        B.chunkft_wgrad_adamw_fused(layer, begin, end, Wb, stB[0], stB[1], stB[2], h, ws=ws)
        if record:
            marks[3].record()
            for k, n in enumerate(names):
                ev[n].append((marks[k], marks[k + 1]))

    if args.timeline:
        print(json.dumps(timeline(torch, np, B, dev, layer, begin, end, g, ws, T,
                                  fused=(Wb, stB, B.hparams(step=1, **hp)) if args.timeline == "fused" else None)), flush=True)
        return

    # Settling: from idle the device needs some tens of milliseconds of this load before its clock
    # management holds a steady state (the first handful of steps run fast, the next twenty to thirty
    # 15 - 25 % slow, then the times level off).  These steps are untimed and come before the W warm-up
    # steps; their gradient times are reported as they were (settling) so the transient is on record.
    settle_us = []
    n_settle = max(args.settle_steps, 0)
    for i in range(n_settle):
        step(i, True)
    torch.cuda.synchronize()
    if n_settle:
        settle_us = [round(a.elapsed_time(b) * 1e3, 1) for a, b in ev["wgrad"]]
        for n in names:
            ev[n].clear()
    for i in range(args.warmup):
        step(n_settle + i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(n_settle + args.warmup + i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms = {n: float(np.mean([a.elapsed_time(b) for a, b in ev[n]])) for n in names}
    ms_med = {n: float(np.median([a.elapsed_time(b) for a, b in ev[n]])) for n in names}

    # the fused call on chunk arrays as torch allocates them (256-byte aligned, whatever `begin` is)
    stC = fresh_state(aligned=False)
    pairs = []
    for i in range(args.warmup + args.steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.chunkft_wgrad_adamw_fused(layer, begin, end, Wb, stC[0], stC[1], stC[2], B.hparams(step=i + 1, **hp), ws=ws)
        b.record()
        if i >= args.warmup:
            pairs.append((a, b))
    torch.cuda.synchronize()
    fused_dense_ms = float(np.mean([a.elapsed_time(b) for a, b in pairs]))
    del stC

    # what the matrix cores sustain on this device when fed from registers alone
    ceil_const = B.chunkft_calib_mfma_bf16(False)
    ceil_rand = B.chunkft_calib_mfma_bf16(True)
    ceil_rand16 = B.chunkft_calib_mfma_bf16_shape(16, True)

    flops = 2.0 * T * E
    R = (end - 1) // case.n_in - begin // case.n_in + 1

    # yardstick, not part of the path: the vendor library's GEMM (torch.mm) on the same operands,
    # the dY columns of the chunk's rows transposed times X, with a bf16 result (half the store traffic)
    r_first = begin // case.n_in

    def lib_gemm_ms(A):
        pairs = []
        for i in range(25):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            torch.mm(A.t(), X)
            b.record()
            if i >= 5:
                pairs.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in pairs]))

    def pair_floor_us(fn):
        pairs = []
        for i in range(60):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            if i >= 10:
                pairs.append((a, b))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in pairs])) * 1e3

    tiny = torch.zeros(64, device=dev)
    floor_empty_us = pair_floor_us(lambda: None)
    floor_tiny_us = pair_floor_us(lambda: tiny.add_(1.0))

    # the plain gradient in a loop of its own, as the yardstick below is timed (operands still in the caches
    # from the call before; in the step loop above 2 GB of optimizer traffic pass between two gradient calls)
    pairs = []
    for i in range(25):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.chunkft_chunk_wgrad(layer, begin, end, g, ws=ws)
        b.record()
        if i >= 5:
            pairs.append((a, b))
    torch.cuda.synchronize()
    wgrad_loop_ms = float(np.median([a.elapsed_time(b) for a, b in pairs]))

    # yardstick for the AdamW pass: a plain streaming kernel of the library over the same number of bytes
    # (half read, half written), settled the same way
    n_copy = int(30.0 * E / 2 / 4)
    src = torch.randn(n_copy, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(80):
        torch.mul(src, 1.0, out=dst)
    pairs = []
    for i in range(20):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        torch.mul(src, 1.0, out=dst)
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    lib_copy_stream_ms = float(np.median([a.elapsed_time(b) for a, b in pairs]))
    del src, dst

    R_even = E // case.n_in
    try:
        lib_view_ms = lib_gemm_ms(dY[:, r_first:r_first + R])                  # the chunk's own row span, as it lies in dY
        lib_copy_ms = lib_gemm_ms(dY[:, r_first:r_first + R_even].contiguous())  # E / in whole rows, packed
    except RuntimeError as ex:                                                   # the yardstick must not cost the result
        print(f"bench.py: library GEMM yardstick failed: {ex}", file=sys.stderr)
        lib_view_ms = lib_copy_ms = float("nan")
    wgrad_bytes = 2.0 * T * case.n_in + 2.0 * T * R + 4.0 * E        # X once, dY columns once, g once
    adamw_bytes = 30.0 * E                                            # g 4 + state 24 + bf16 W 2
    fused_bytes = 26.0 * E + 2.0 * T * (case.n_in + R)
    wgrad_tflops = flops / (ms["wgrad"] * 1e-3) / 1e12
    adamw_gbps = adamw_bytes / (ms["adamw"] * 1e-3) / 1e9
    fused_bound_ms = max(flops / (PEAK_BF16_TFLOPS * 1e12), fused_bytes / (PEAK_HBM_GBPS * 1e9)) * 1e3

    out = {
        "metric": "chunk wgrad TFLOP/s (% MFMA peak) + AdamW GB/s (% HBM) at Llama-3-8B shapes",
        "value": round(wgrad_tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: Llama-3-8B up_proj 14336x4096 bf16, T=1024, chunk of 32Mi elements "
                        f"[{begin},{end}) (row span {R}), fp32 master/m/v for the chunk only",
            "step": "plan_cycle + chunk_wgrad + adamw_chunk + wgrad_adamw_fused",
            "split_k": S,
            "settling": {"what": "untimed steps before the warm-up steps until the clock management holds a steady "
                                 "state under this load; the gradient call's time in each of them, in order",
                         "steps": n_settle,
                         "wgrad_us_steps_2_to_9": settle_us[1:9],
                         "wgrad_us_slowest_after_the_first": max(settle_us[1:]) if len(settle_us) > 1 else None,
                         "wgrad_us_last_8": settle_us[-8:]},
            "chunk_arrays": "g, master, m, v at the 128-byte phase of the tensor rows (element i of an array "
                            "has the address phase of element begin + i of W); master, m, v cut from one "
                            "allocation, a whole number of MiB + 256 KiB apart (binding.chunk_state)",
        },
        "wgrad": {"ms": round(ms["wgrad"], 4), "ms_median": round(ms_med["wgrad"], 4),
                  "tflops": round(wgrad_tflops, 2), "pct_mfma_peak": round(100 * wgrad_tflops / PEAK_BF16_TFLOPS, 2),
                  "ms_median_in_a_loop_of_its_own": round(wgrad_loop_ms, 4)},
        "adamw": {"ms": round(ms["adamw"], 4), "ms_median": round(ms_med["adamw"], 4),
                  "gbps": round(adamw_gbps, 1), "pct_hbm_peak": round(100 * adamw_gbps / PEAK_HBM_GBPS, 2)},
        "fused": {"ms": round(ms["fused"], 4), "ms_median": round(ms_med["fused"], 4),
                  "bound": "hbm", "bound_ms": round(fused_bound_ms, 4),
                  "frac_of_bound": round(fused_bound_ms / ms["fused"], 4),
                  "gbps": round(fused_bytes / (ms["fused"] * 1e-3) / 1e9, 1),
                  "tflops": round(flops / (ms["fused"] * 1e-3) / 1e12, 2),
                  "traffic": MEASURED_TRAFFIC["fused"], "algorithmic_bytes": fused_bytes,
                  "ms_with_arrays_as_allocated": round(fused_dense_ms, 4)},
        "roofline": {"kernel": "wgrad_mfma_kernel (chunkft_chunk_wgrad)", "bound": "mfma",
                     "achieved": round(wgrad_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(wgrad_tflops / PEAK_BF16_TFLOPS, 4), "traffic": MEASURED_TRAFFIC["wgrad"],
                     "algorithmic_bytes": wgrad_bytes,
                     "event_pair_floor_us": {"what": "what the same pair of events reads around nothing and around "
                                                     "a 64-element kernel: part of every figure here",
                                             "nothing": round(floor_empty_us, 2), "tiny_kernel": round(floor_tiny_us, 2)},
                     "library_gemm": {
                         "what": "yardstick only, not part of the path: torch.mm (the vendor library's GEMM) of the "
                                 "transposed dY columns with X, bf16 result instead of fp32, median of 20",
                         "chunk_rows_as_they_lie": None if lib_view_ms != lib_view_ms else {
                             "rows": R, "ms": round(lib_view_ms, 4),
                             "tflops": round(2.0 * T * R * case.n_in / (lib_view_ms * 1e-3) / 1e12, 2)},
                         "whole_rows_packed": None if lib_copy_ms != lib_copy_ms else {
                             "rows": R_even, "ms": round(lib_copy_ms, 4),
                             "tflops": round(2.0 * T * R_even * case.n_in / (lib_copy_ms * 1e-3) / 1e12, 2)}},
                     "mfma_only_measured": {
                         "what": "32x32x16 bf16 MFMAs issued from registers, nothing else, two waves per SIMD "
                                 "(chunkft_calib_mfma_bf16): the sustained clock, hence the reachable rate, "
                                 "drops when the operands are random bit patterns as in a real contraction",
                         "constant_operands": {"tflops": round(ceil_const[0], 1), "shader_mhz": round(ceil_const[1])},
                         "random_operands": {"tflops": round(ceil_rand[0], 1), "shader_mhz": round(ceil_rand[1])},
                         "frac_of_random_operand_rate": round(wgrad_tflops / ceil_rand[0], 4),
                         "random_operands_16x16x32": {"tflops": round(ceil_rand16[0], 1),
                                                      "shader_mhz": round(ceil_rand16[1]),
                                                      "frac_of_this_rate": round(wgrad_tflops / ceil_rand16[0], 4),
                                                      "what": "the other bf16 shape draws less power and holds "
                                                              "a higher clock; the gradient kernel's 256 x 256 "
                                                              "tile, which this workload takes, issues it"}}},
        "roofline_adamw": {"kernel": "elementwise_kernel (chunkft_adamw_chunk)", "bound": "hbm",
                           "achieved": round(adamw_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                           "frac": round(adamw_gbps / PEAK_HBM_GBPS, 4), "traffic": MEASURED_TRAFFIC["adamw"],
                           "algorithmic_bytes": adamw_bytes,
                           "library_copy": {"what": "yardstick only: torch.mul(src, 1.0, out=dst) over the same number "
                                                    "of bytes, half read and half written, median of 20",
                                            "ms": round(lib_copy_stream_ms, 4),
                                            "gbps": round(2.0 * n_copy * 4 / (lib_copy_stream_ms * 1e-3) / 1e9, 1)}},
    }

    if not args.no_per_config:
        out["per_config"] = per_config(torch, B, WL, dev, dict(WL.HPARAMS), cfg2=(layer, begin, end, W, g, ws))

    if args.sweep:
        out["sweep"] = sweep(torch, B, dev, dict(WL.HPARAMS))

    if args.stream_state:
        out["streamed_state"] = streamed_state(torch, B, dev, layer, begin, end, Wb, h_for=lambda n: B.hparams(step=n, **hp), ws=ws)

    if args.plan_sweep:
        out["plan_sweep"] = plan_sweep(B)

    if args.block_cycle:
        out["block_cycle"] = block_cycle(torch, B, dev, dict(WL.HPARAMS))

    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)          # one element-wise kernel: 4 B read + 4 B written per element
        torch.cuda.synchronize()
        out["copy_probe"] = {"kernel": "torch.mul(src, 1.0, out=dst)", "read_bytes": src.numel() * 4,
                             "write_bytes": src.numel() * 4}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case, begin, end, hp)
    print(json.dumps(out), flush=True)


def timeline(torch, np, B, dev, layer, begin, end, g, ws, T, fused=None):
    """Phase times of every workgroup of the plain gradient's MFMA kernel at the benchmark workload, from
    the diagnostic build of the library.  Times are the 100 MHz constant counter (10 ns steps)."""
    L = B.load_timeline_library()
    cap = 1 << 16
    buf = torch.zeros(cap * 8, dtype=torch.int64, device=dev)
    def call():
        if fused is None:
            B.chunkft_chunk_wgrad(layer, begin, end, g, ws=ws)
        else:
            W, st, h = fused
            B.chunkft_wgrad_adamw_fused(layer, begin, end, W, st[0], st[1], st[2], h, ws=ws)

    with B.use_library(L):
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        L.chunkft_timeline_buffer(buf.data_ptr(), buf.numel() * 8)
        call()
        torch.cuda.synchronize()
        L.chunkft_timeline_buffer(None, 0)
    t = buf.cpu().numpy().reshape(cap, 8)
    t = t[t[:, 0] != 0]
    us = lambda ticks: ticks / 100.0
    t0 = t[:, 0].min()
    start, frag, loop_end, done = (us(t[:, k] - t0) for k in range(4))
    where = t[:, 4]
    hw = where & 0xffffffff
    # HW_ID: compute unit [11:8], shader array [12], shader engine [15:13]; XCC_ID [3:0] in the upper word
    cu = ((where >> 32) & 0xf) * 4096 + ((hw >> 13) & 7) * 64 + ((hw >> 12) & 1) * 16 + ((hw >> 8) & 0xf)
    span = float(done.max())
    units = np.unique(cu)

    def stats(x):
        return {"mean": round(float(x.mean()), 2), "p10": round(float(np.quantile(x, 0.1)), 2),
                "median": round(float(np.median(x)), 2), "p90": round(float(np.quantile(x, 0.9)), 2)}

    # per compute unit: how long at least one / two of its workgroups are in their MFMA loop
    one_loop, two_loops, first_start, last_done, per_cu = [], [], [], [], []
    for u in units:
        sel = cu == u
        ev = sorted([(a, 1) for a in frag[sel]] + [(b, -1) for b in loop_end[sel]])
        depth, prev, t1, t2 = 0, 0.0, 0.0, 0.0
        for when, d in ev:
            if depth >= 1: t1 += when - prev
            if depth >= 2: t2 += when - prev
            depth += d
            prev = when
        one_loop.append(t1); two_loops.append(t2)
        first_start.append(start[sel].min()); last_done.append(done[sel].max()); per_cu.append(int(sel.sum()))
    one_loop, two_loops = np.array(one_loop), np.array(two_loops)
    order = np.argsort(start)
    rounds = {}
    n_first = len(units) * (2 if len(t) >= 2 * len(units) else 1)
    for name, sel in (("workgroups started first on their place", order[:n_first]), ("workgroups started later", order[n_first:])):
        if len(sel):
            rounds[name] = {"count": int(len(sel)), "start_us": stats(start[sel]),
                            "first_fragments_after_us": stats((frag - start)[sel]),
                            "loop_us": stats((loop_end - frag)[sel]), "epilogue_us": stats((done - loop_end)[sel])}
    return {"kernel": "wgrad_mfma_kernel, %s of the benchmark workload (libchunkft_timeline.so)" % (
                "plain gradient" if fused is None else "fused call"),
            "workgroups": int(len(t)), "compute_units_seen": int(len(units)), "workgroups_per_compute_unit": stats(np.array(per_cu)),
            "span_us": round(span, 2),
            "phase_us_per_workgroup": {"first_fragments_after_start": stats(frag - start), "loop": stats(loop_end - frag),
                                       "epilogue": stats(done - loop_end), "whole": stats(done - start)},
            "by_round": rounds,
            "per_compute_unit_us": {"first_start": stats(np.array(first_start)), "last_end": stats(np.array(last_done)),
                                    "some_workgroup_in_its_loop": stats(one_loop), "two_workgroups_in_their_loops": stats(two_loops),
                                    "no_workgroup_in_its_loop": stats(span - one_loop)},
            "mfma_flops_time_at_2.5_PFLOPs_us": round(2.0 * T * (end - begin) / 2.5e15 * 1e6, 2)}


def llama3_8b_tensors(B):
    """Every trainable tensor of a Llama-3-8B-shaped model in model order: (rows, cols, dtype, kind)."""
    h, kv, ff, vocab, n_layers = 4096, 1024, 14336, 128256, 32
    tensors = [(vocab, h, B.BF16, B.EMBEDDING)]
    for _ in range(n_layers):
        tensors += [(1, h, B.BF16, B.RMSNORM), (h, h, B.BF16, B.LINEAR), (kv, h, B.BF16, B.LINEAR),
                    (kv, h, B.BF16, B.LINEAR), (h, h, B.BF16, B.LINEAR), (1, h, B.BF16, B.RMSNORM),
                    (ff, h, B.BF16, B.LINEAR), (ff, h, B.BF16, B.LINEAR), (h, ff, B.BF16, B.LINEAR)]
    tensors += [(1, h, B.BF16, B.RMSNORM), (vocab, h, B.BF16, B.LINEAR)]
    # layer-wise partition for contrast: embedding | each decoder layer | final norm + head
    groups = [[0]] + [list(range(1 + 9 * i, 10 + 9 * i)) for i in range(n_layers)] + [[len(tensors) - 2, len(tensors) - 1]]
    return tensors, groups


def plan_sweep(B, tensors=None, layer_groups=None, budgets=None):
    """The planner on every tensor of a model in model order (default: Llama-3-8B shapes), with the
    training cost per element (parameter + fp32 gradient, master, m, v).  For each budget and
    planner variant: chunks produced, the largest deviation of a chunk's cost from the mean (the
    imbalance of the paper's jitter analysis), the jitter (max - min) / mean of the step memory
    2 M + B(C_k), activations left out, and the analysis' bound on it -- all four from
    chunkft_plan_stats; the same for a partition by layer, which is what layer-wise rotating
    methods use.  Host only."""
    if tensors is None:
        tensors, layer_groups = llama3_8b_tensors(B)
    elem = {B.BF16: 2, B.F32: 4}
    numel = [r * c for r, c, _, _ in tensors]
    resident = sum(n * elem[d] for n, (_, _, d, _) in zip(numel, tensors))       # the 2M of the analysis
    cost = [n * (elem[d] + 16) for n, (_, _, d, _) in zip(numel, tensors)]
    total_cost = sum(cost)

    def row(label, name, chunks):
        st = B.chunkft_plan_stats(chunks, resident)
        return {"budget": label, "planner": name, "chunks": st["n_chunks"], "max_cost_bytes": st["max_cost_bytes"],
                "imbalance_bytes": st["imbalance_bytes"], "jitter": st["jitter"], "jitter_bound": st["jitter_bound"]}

    rows = []
    if budgets is None:
        budgets = [("%d chunks" % K, -(-total_cost // K) + (-(-(-total_cost // K))) % 18) for K in (7, 32, 100)]
        budgets += [("%d GiB" % gib, gib << 30) for gib in (1, 2, 4, 8)]
    for label, budget in budgets:
        for name, flags in (("greedy", B.PLAN_TRAINING_COST), ("balanced", B.PLAN_TRAINING_COST | B.PLAN_BALANCED),
                            ("greedy, cuts between groups of 8 rows", B.PLAN_TRAINING_COST | B.PLAN_ROWS8)):
            _, chunks, _ = B.chunkft_plan_cycle(tensors, budget, flags)
            rows.append(row(label, name, chunks))
    if layer_groups:
        by_layer = [(0, 0, sum(numel[t] for t in grp), sum(cost[t] for t in grp)) for grp in layer_groups]
        rows.append(row("-", "one partition per layer (for contrast)", by_layer))
    return {"model": "%d tensors, %.3f G parameters, %d resident bytes" % (len(tensors), sum(numel) / 1e9, resident),
            "rows": rows}


def streamed_state(torch, B, dev, layer, begin, end, W, h_for, ws):
    """Algorithm 1's streaming on this workload: K = 3 chunks of E elements whose master/m/v live in
    pinned host memory, interval 4, two device buffer sets.  Every visit runs 4 fused updates on the
    same layer range (the kernels' cost is what matters here, not which rows they touch) while the
    next chunk's 12 E bytes come in and the previous chunk's go out.  Reports the wall time per
    visit against the time of the copies alone and of the kernels alone."""
    E, K, interval, cycles = end - begin, 3, 4, 2
    host = [tuple(torch.zeros(E, dtype=torch.float32).pin_memory() for _ in range(3)) for _ in range(K)]
    sets = [tuple(torch.zeros(E, dtype=torch.float32, device=dev) for _ in range(3)) for _ in range(2)]
    mover = B.Mover()
    n_steps = cycles * K * interval

    def run(stream_copies, kernels):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        visit = -1
        for t in range(n_steps):
            k, load, off, n = B.chunkft_schedule_at(t, K, interval)
            if load:
                visit += 1
                if stream_copies:
                    if visit == 0:
                        mover.load(sets[0], host[k], E)
                    mover.await_load()
                    mover.load(sets[(visit + 1) % 2], host[(k + 1) % K], E)
            cur = sets[visit % 2]
            if kernels:
                B.chunkft_wgrad_adamw_fused(layer, begin, end, W, cur[0], cur[1], cur[2], h_for(n), ws=ws)
            if off and stream_copies:
                mover.offload(host[k], cur, E)
        torch.cuda.synchronize()
        if stream_copies:
            mover.sync()
        return (time.perf_counter() - t0) / (cycles * K)

    run(True, True)                                   # warm-up
    both = run(True, True)
    copies = run(True, False)
    kernels = run(False, True)
    mover.close()
    per_visit_bytes = 2 * 12.0 * E                    # 12 E in, 12 E out
    return {"chunks": K, "interval": interval, "chunk_elements": E,
            "ms_per_visit": round(both * 1e3, 3), "ms_copies_alone": round(copies * 1e3, 3),
            "ms_kernels_alone": round(kernels * 1e3, 3),
            "host_link_gbps_each_way": round(12.0 * E / copies / 1e9, 1),
            "overlap_efficiency": round(max(copies, kernels) / both, 4),
            "note": "bound by the host link: a visit moves %.0f MB, its kernels take %.2f ms" % (per_visit_bytes / 1e6, kernels * 1e3)}


def block_cycle(torch, B, dev, hp, reps=10, graph=True):
    """One cycle over the nine tensors of a Llama-3-8B block (configs[2]): plan with a 256 MiB budget,
    then per chunk one fused call per segment on one stream (a chunk may cross tensors), median of
    `reps`.  The state of a chunk is kept as one set of arrays per segment, each in the recommended
    layout."""
    T = 1024
    gen = torch.Generator(device=dev)
    gen.manual_seed(211773)
    shapes = [("q", 4096, 4096, "h"), ("k", 1024, 4096, "h"), ("v", 1024, 4096, "h"), ("o", 4096, 4096, "a"),
              ("gate", 14336, 4096, "n"), ("up", 14336, 4096, "n"), ("down", 4096, 14336, "f"),
              ("norm1", 1, 4096, "x1"), ("norm2", 1, 4096, "x2")]
    inputs = {}

    def x_for(key, width):
        if key not in inputs:
            inputs[key] = torch.randn(T, width, device=dev, generator=gen).to(torch.bfloat16)
        return inputs[key]

    layers, Ws, tensors = [], [], []
    for name, out_f, in_f, xkey in shapes:
        X = x_for(xkey, in_f)
        dY = (torch.randn(T, out_f if out_f > 1 else in_f, device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
        kind = B.LINEAR if out_f > 1 else B.VECTOR
        layers.append(B.make_layer(kind, X, dY, out_f, in_f))
        Ws.append((torch.randn(out_f * in_f, device=dev, generator=gen) * 0.02).to(torch.bfloat16))
        tensors.append((out_f, in_f, B.BF16, kind))
        inputs[name + "_dY"] = dY                         # keeps the tensor alive
    _, chunks, segs = B.chunkft_plan_cycle(tensors, 256 << 20)
    h = B.hparams(step=1, **hp)
    rows = []
    for k, (s0, s1, numel, cost) in enumerate(chunks):
        # one set of state arrays per segment, each at the line phase of its tensor rows
        work = []
        for (t, b, e, off) in segs[s0:s1]:
            nws = B.chunkft_workspace_bytes(layers[t], b, e)
            ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
            state = B.chunk_state(e - b, b, dev)
            state[0].copy_(Ws[t][b:e]); state[1].zero_(); state[2].zero_()
            work.append((t, b, e, state, ws))

        def per_segment_calls():
            for (t, b, e, state, ws) in work:
                B.chunkft_wgrad_adamw_fused(layers[t], b, e, Ws[t], state[0], state[1], state[2], h, ws=ws)

        group = B.GroupCall([(layers[t], b, e, Ws[t], state[0], state[1], state[2]) for (t, b, e, state, ws) in work],
                            device=dev)

        def grouped_call():
            group(h)

        ms_seg = _median_ms(torch, per_segment_calls, reps=reps)
        ms = _median_ms(torch, grouped_call, reps=reps)
        row = {"chunk": k, "elements": numel, "launch": "chunkft_wgrad_adamw_fused_group: one call for the chunk",
               "ms": round(ms, 4), "ms_per_segment_calls": round(ms_seg, 4)}
        if graph:
            # the same call replayed from a captured HIP graph (the entry points only enqueue kernels)
            stream = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                with torch.cuda.graph(g, stream=stream):
                    grouped_call()
            torch.cuda.synchronize()
            row["ms_graph_replay"] = round(_median_ms(torch, g.replay, reps=reps), 4)
            del g
        seg_rows = []
        for (t, b, e, state, ws) in work:          # each segment by itself, back to back with itself
            alone = _median_ms(torch, lambda: B.chunkft_wgrad_adamw_fused(layers[t], b, e, Ws[t], state[0], state[1],
                                                                          state[2], h, ws=ws), reps=max(4, reps // 2))
            in_f = shapes[t][2]
            seg_rows.append({"tensor": shapes[t][0], "elements": e - b, "in": in_f if shapes[t][1] > 1 else 0,
                             "rows": (e - 1) // in_f - b // in_f + 1,
                             "split_k": B.chunkft_split_k(layers[t], b, e), "ms_alone": round(alone, 4)})
        row["segments"] = seg_rows
        row["ns_per_kilo_element"] = round(ms * 1e6 / (numel / 1e3), 3)
        row["tflops"] = round(2.0 * T * numel / ms / 1e9, 1)
        row["state_gbps"] = round(26.0 * numel / ms / 1e6, 1)
        rows.append(row)
    return {"T": T, "budget_MiB": 256, "tensors": [s[0] for s in shapes], "chunks": rows,
            "cycle_ms": round(sum(r["ms"] for r in rows), 4),
            "cycle_ms_per_segment_calls": round(sum(r["ms_per_segment_calls"] for r in rows), 4)}


def _median_ms(torch, fn, reps=10, warm=2, settle_ms=30.0):
    """Median event time of `reps` calls issued back to back, after at least `warm` calls and `settle_ms`
    of the same load (the device's clocks need that long from idle or from a lighter load, see main())."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); fn(); b.record(); b.synchronize()
    first = max(a.elapsed_time(b), 1e-3)
    for _ in range(max(warm - 1, min(int(settle_ms / first), 400))):
        fn()
    pairs = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); fn(); b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ts = [a.elapsed_time(b) for a, b in pairs]
    return sorted(ts)[len(ts) // 2]


def _fused_bound_ms(T, segs):
    """Governing bound of fused calls on segments (elements, in, row span): the larger of the MFMA time
    of 2 T E flops and the HBM time of 26 E bytes of state plus the operands read once."""
    fl = sum(2.0 * T * e for e, _, _ in segs)
    by = sum(26.0 * e + 2.0 * T * (n_in + rows) for e, n_in, rows in segs)
    t_mfma, t_hbm = fl / (PEAK_BF16_TFLOPS * 1e12) * 1e3, by / (PEAK_HBM_GBPS * 1e9) * 1e3
    return max(t_mfma, t_hbm), ("mfma" if t_mfma >= t_hbm else "hbm"), fl, by


def per_config(torch, B, WL, dev, hp, cfg2):
    """Every configuration of the task's list beside the headline one, timed on device-generated
    operands of its shapes and value scales (X ~ N(0,1), dY ~ N(0,1e-3), configs[4]: 90 % of the token
    rows N(0,1e-4), 10 % N(0,1e-2)), median of 10 calls between HIP events on the call's stream.
    Chunk arrays in the recommended layout; state sets are rotated where one set would stay in the
    256 MB last-level cache between two calls."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(211775)
    h1 = B.hparams(step=1, **hp)
    rows = []

    def operands(out_f, in_f, T, dy_scale):
        X = torch.randn(T, in_f, device=dev, generator=gen).to(torch.bfloat16)
        dY = (torch.randn(T, out_f, device=dev, generator=gen) * dy_scale).to(torch.bfloat16)
        W = (torch.randn(out_f * in_f, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
        return X, dY, W

    def rowspan(b, e, n_in):
        return (e - 1) // n_in - b // n_in + 1

    # ---- configs[1] again: the fused call on warm moments (a later visit of the chunk), and the AdamW
    # pass on a gradient that is not in any cache (four gradient / state sets in rotation)
    layer, begin, end, W, g, ws = cfg2
    E = end - begin
    sets = []
    for _ in range(4):
        st = B.chunk_state(E, begin, dev, count=4)
        st[0].copy_(W[begin:end]); st[1].normal_(0.0, 1e-3, generator=gen); st[2].uniform_(1e-7, 1e-6, generator=gen)
        st[3].normal_(0.0, 3e-2, generator=gen)
        sets.append(st)
    turn = [0]

    def warm_fused():
        turn[0] += 1
        m_, a_, v_, _ = sets[turn[0] % 4]
        B.chunkft_wgrad_adamw_fused(layer, begin, end, W, m_, a_, v_, B.hparams(step=2, **hp), ws=ws)

    def cold_adamw():
        turn[0] += 1
        m_, a_, v_, g_ = sets[turn[0] % 4]
        B.chunkft_adamw_chunk(g_, m_, a_, v_, W[begin:end], E, B.hparams(step=2, **hp))

    t = _median_ms(torch, warm_fused, reps=12)
    bound, which, fl, by = _fused_bound_ms(1024, [(E, 4096, rowspan(begin, end, 4096))])
    rows.append({"config": 1, "case": "fused call, warm moments (step 2), state sets rotated", "ms": round(t, 4),
                 "tflops": round(fl / t / 1e9, 1), "gbps": round(by / t / 1e6, 1), "bound": which,
                 "frac_of_bound": round(bound / t, 4)})
    t = _median_ms(torch, cold_adamw, reps=12)
    rows.append({"config": 1, "case": "AdamW pass, gradient and state not in any cache (four sets rotated)",
                 "ms": round(t, 4), "gbps": round(30.0 * E / t / 1e6, 1), "bound": "hbm",
                 "frac_of_bound": round(30.0 * E / t / 1e6 / PEAK_HBM_GBPS, 4)})
    del sets
    torch.cuda.empty_cache()

    # ---- configs[2]: the transformer block, one cycle under a 256 MiB budget
    blk = block_cycle(torch, B, dev, hp, reps=6, graph=False)
    for ch in blk["chunks"]:
        segs = [(sg["elements"], sg["in"], sg["rows"]) for sg in ch["segments"] if sg["in"] > 0]
        bound, which, fl, by = _fused_bound_ms(blk["T"], segs)
        rows.append({"config": 2, "case": "block cycle, 256 MiB budget, chunk %d: %s" % (
                         ch["chunk"], " ".join("%s[%d]" % (sg["tensor"], sg["elements"]) for sg in ch["segments"])),
                     "launch": ch["launch"], "ms": ch["ms"], "ms_one_call_per_segment": ch["ms_per_segment_calls"],
                     "tflops": round(fl / ch["ms"] / 1e9, 1), "gbps": round(by / ch["ms"] / 1e6, 1), "bound": which,
                     "frac_of_bound": round(bound / ch["ms"], 4)})

    # ---- configs[3]: 70B-shaped MLP, T = 8192
    T, hdim, ff = 8192, 8192, 28672
    ops = {0: ("gate 28672x8192", ff, hdim) + operands(ff, hdim, T, 1e-3),
           1: ("down 8192x28672", hdim, ff) + operands(hdim, ff, T, 1e-3)}
    chunks = WL.config4_chunks(ff * hdim, hdim, ff * hdim)
    off = WL.draw_offset(WL.rng_for(4, 2), ff * hdim, 64 << 20, hdim)
    cases = [("gate, 128 MiB chunk at a seeded mid-row offset", [(0, off, off + (64 << 20))]),
             ("128 MiB chunk at the seeded offset of the [gate | down] space", chunks["seeded"]),
             ("128 MiB chunk straddling gate -> down", chunks["straddling"]),
             ("1 GiB budget: gate and down whole (896 MiB)", chunks["whole"])]
    for label, segs in cases:
        work = []
        for (ti, b, e) in segs:
            name, out_f, in_f, X, dY, Wt = ops[ti]
            lay = B.make_layer(B.LINEAR, X, dY, out_f, in_f)
            st = B.chunk_state(e - b, b, dev)
            st[0].copy_(Wt[b:e]); st[1].zero_(); st[2].zero_()
            gg = B.chunk_array(e - b, b, dev)
            nws = B.chunkft_workspace_bytes(lay, b, e)
            wsp = torch.empty(max(nws // 4, 1), dtype=torch.float32, device=dev) if nws else None
            work.append((lay, b, e, Wt, st, gg, wsp, in_f, B.chunkft_split_k(lay, b, e)))

        def fused_all():
            for (lay, b, e, Wt, st, gg, wsp, _, _) in work:
                B.chunkft_wgrad_adamw_fused(lay, b, e, Wt, st[0], st[1], st[2], h1, ws=wsp)

        def wgrad_all():
            for (lay, b, e, Wt, st, gg, wsp, _, _) in work:
                B.chunkft_chunk_wgrad(lay, b, e, gg, ws=wsp)

        tf_, tw_ = _median_ms(torch, fused_all, reps=6), _median_ms(torch, wgrad_all, reps=6)
        bound, which, fl, by = _fused_bound_ms(T, [(e - b, in_f, rowspan(b, e, in_f)) for (_, b, e, _, _, _, _, in_f, _) in work])
        rows.append({"config": 3, "case": label, "segments": len(work), "split_k": [w[8] for w in work],
                     "fused_ms": round(tf_, 4), "fused_tflops": round(fl / tf_ / 1e9, 1), "bound": which,
                     "frac_of_bound": round(bound / tf_, 4), "wgrad_ms": round(tw_, 4),
                     "wgrad_tflops": round(fl / tw_ / 1e9, 1),
                     "wgrad_pct_mfma_peak": round(100 * fl / tw_ / 1e9 / PEAK_BF16_TFLOPS, 2)})
        del work
        torch.cuda.empty_cache()
    del ops
    torch.cuda.empty_cache()

    # ---- configs[4]: lm_head shape, T = 4096, per chunk size
    T, vocab, dim = 4096, 128256, 4096
    X = torch.randn(T, dim, device=dev, generator=gen).to(torch.bfloat16)
    scale = torch.where(torch.rand(T, 1, device=dev, generator=gen) < 0.1, 1e-2, 1e-4)
    dY = (torch.randn(T, vocab, device=dev, generator=gen) * scale).to(torch.bfloat16)
    Wt = (torch.randn(vocab * dim, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
    lay = B.make_layer(B.LINEAR, X, dY, vocab, dim)

    class _Shape:                        # what config5_ranges needs of a layer
        numel, n_in = vocab * dim, dim

    for mib, (b, e) in zip(WL.CONFIG5_CHUNK_MIB, WL.config5_ranges(_Shape)):
        E5 = e - b
        n_sets = max(1, min(16, int((1 << 30) // (16 * E5))))
        sets = []
        for _ in range(n_sets):
            st = B.chunk_state(E5, b, dev, count=4)
            st[0].copy_(Wt[b:e]); st[1].zero_(); st[2].zero_()
            sets.append(st)
        nws = B.chunkft_workspace_bytes(lay, b, e)
        wsp = torch.empty(max(nws // 4, 1), dtype=torch.float32, device=dev) if nws else None
        turn = [0]

        def fused5():
            turn[0] += 1
            m_, a_, v_, _ = sets[turn[0] % n_sets]
            B.chunkft_wgrad_adamw_fused(lay, b, e, Wt, m_, a_, v_, h1, ws=wsp)

        def wgrad5():
            turn[0] += 1
            B.chunkft_chunk_wgrad(lay, b, e, sets[turn[0] % n_sets][3], ws=wsp)

        reps = max(10, 2 * n_sets)
        tf_, tw_ = _median_ms(torch, fused5, reps=reps), _median_ms(torch, wgrad5, reps=reps)
        bound, which, fl, by = _fused_bound_ms(T, [(E5, dim, rowspan(b, e, dim))])
        rows.append({"config": 4, "case": "lm_head 128256x4096, %d MiB chunk at a seeded mid-row offset" % mib,
                     "split_k": B.chunkft_split_k(lay, b, e), "state_sets_rotated": n_sets,
                     "fused_ms": round(tf_, 4), "fused_tflops": round(fl / tf_ / 1e9, 1),
                     "fused_gbps": round(by / tf_ / 1e6, 1), "bound": which, "frac_of_bound": round(bound / tf_, 4),
                     "wgrad_ms": round(tw_, 4), "wgrad_tflops": round(fl / tw_ / 1e9, 1),
                     "wgrad_pct_mfma_peak": round(100 * fl / tw_ / 1e9 / PEAK_BF16_TFLOPS, 2)})
        del sets
        torch.cuda.empty_cache()
    return rows


def sweep(torch, B, dev, hp):
    import numpy as np

    """Plain and fused call on device-generated Gaussian operands of other shapes (same recipe:
    X ~ N(0,1), dY ~ N(0,1e-3), two-scale token rows for the lm_head shape), median of 10."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(211770)
    rows = []

    def timed(fn, reps=10):
        for _ in range(2):
            fn()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); b.synchronize()
            ts.append(a.elapsed_time(b))
        return sorted(ts)[len(ts) // 2]

    def one(name, out_f, in_f, T, E, dy_scale, x_scale=1.0, rows8=False):
        X = (torch.randn(T, in_f, device=dev, generator=gen) * x_scale).to(torch.bfloat16)
        dY = (torch.randn(T, out_f, device=dev, generator=gen) * dy_scale).to(torch.bfloat16)
        W = (torch.randn(out_f * in_f, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
        begin = (out_f * in_f - E) // 2 + 37
        begin -= 1 if begin % in_f == 0 else 0
        if rows8:          # a chunk as the planner cuts it with CHUNKFT_PLAN_ROWS8
            begin = begin // (8 * in_f) * (8 * in_f)
        end = begin + E
        layer = B.make_layer(B.LINEAR, X, dY, out_f, in_f)
        nws = B.chunkft_workspace_bytes(layer, begin, end)
        ws = torch.empty(max(nws // 4, 1), dtype=torch.float32, device=dev) if nws else None
        # A small chunk's state would stay in the 256 MB last-level cache from one timed call to
        # the next: rotate over enough distinct sets of g / master / m / v that each call finds
        # its set evicted (about 1 GB between two uses of the same set).
        n_sets = max(1, min(16, int((1 << 30) // (16 * E))))
        gs = [B.chunk_array(E, begin, dev) for _ in range(n_sets)]
        sets = []
        zero = torch.zeros((), dtype=torch.float32, device=dev)
        for _ in range(n_sets):
            st = B.chunk_state(E, begin, dev)
            st[0].copy_(W[begin:end]); st[1].zero_(); st[2].zero_()
            sets.append(st)
        h = B.hparams(step=1, **hp)
        turn = [0]

        def call_wgrad():
            turn[0] += 1
            B.chunkft_chunk_wgrad(layer, begin, end, gs[turn[0] % n_sets], ws=ws)

        def call_fused():
            turn[0] += 1
            master, m, v = sets[turn[0] % n_sets]
            B.chunkft_wgrad_adamw_fused(layer, begin, end, W, master, m, v, h, ws=ws)

        t_w = timed(call_wgrad, reps=max(10, 2 * n_sets))
        t_f = timed(call_fused, reps=max(10, 2 * n_sets))
        fl = 2.0 * T * E
        R = (end - 1) // in_f - begin // in_f + 1
        bound = max(fl / (PEAK_BF16_TFLOPS * 1e12), (26.0 * E + 2.0 * T * (in_f + R)) / (PEAK_HBM_GBPS * 1e9)) * 1e3
        rows.append({"shape": name, "T": T, "chunk_MiB": E * 2 // (1 << 20), "state_sets_rotated": n_sets,
                     "split_k": B.chunkft_split_k(layer, begin, end),
                     "wgrad_ms": round(t_w, 4), "wgrad_tflops": round(fl / t_w / 1e9, 1),
                     "fused_ms": round(t_f, 4), "fused_tflops": round(fl / t_f / 1e9, 1),
                     "fused_frac_of_bound": round(bound / t_f, 4)})

    for T in (1024, 4096, 8192):
        one("up_proj 14336x4096", 14336, 4096, T, 32 << 20, 1e-3)
    for T in (1024, 4096, 8192):
        one("up_proj 14336x4096, chunk between rows that are multiples of 8", 14336, 4096, T, 32 << 20, 1e-3,
            rows8=True)
    # the same launch on all-zero operands: same instructions, same cycles, but few bits toggle
    # in the matrix cores, so the part holds a higher clock -- the size of the data-dependent
    # clock effect on this kernel (not a performance figure)
    one("up_proj 14336x4096, all-zero operands (clock probe)", 14336, 4096, 1024, 32 << 20, 0.0, x_scale=0.0)
    scale = torch.where(torch.rand(4096, 1, device=dev, generator=gen) < 0.1, 1e-2, 1e-4)
    for mib in (4, 16, 64, 256, 512):
        one("lm_head 128256x4096", 128256, 4096, 4096, mib << 19, scale)

    # embedding table of the same shape (HBM-bound row gather): ids with heavy-tailed frequencies
    vocab, dim, T = 128256, 4096, 4096
    ranks = (torch.exp(torch.rand(T, device=dev, generator=gen) * float(np.log(vocab + 1.0))) - 1.0).long().clamp_(max=vocab - 1)
    ids = torch.randperm(vocab, device=dev, generator=gen)[ranks].contiguous()
    dY = (torch.randn(T, dim, device=dev, generator=gen) * 1e-3).to(torch.bfloat16)
    W = (torch.randn(vocab * dim, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
    for mib in (64, 512):
        E = mib << 19
        begin = (vocab * dim - E) // 2 + 37
        end = begin + E
        layer = B.make_layer(B.EMBEDDING, ids, dY, vocab, dim)
        zero = torch.zeros((), dtype=torch.float32, device=dev)
        g = B.chunk_array(E, begin, dev)
        master, m, v = B.chunk_state(E, begin, dev)
        master.copy_(W[begin:end]); m.zero_(); v.zero_()
        h = B.hparams(step=1, **hp)
        t_w = timed(lambda: B.chunkft_chunk_wgrad(layer, begin, end, g))
        t_f = timed(lambda: B.chunkft_wgrad_adamw_fused(layer, begin, end, W, master, m, v, h))
        t_a = timed(lambda: B.chunkft_chunk_wgrad(layer, begin, end, g, accumulate=True))
        rows.append({"shape": "embedding 128256x4096", "T": T, "chunk_MiB": mib, "bound": "hbm",
                     "wgrad_ms": round(t_w, 4), "wgrad_gbps": round(4.0 * E / t_w / 1e6, 1),
                     "wgrad_accumulate_ms": round(t_a, 4),
                     "fused_ms": round(t_f, 4), "fused_gbps": round(26.0 * E / t_f / 1e6, 1),
                     "fused_frac_of_hbm_peak": round(26.0 * E / t_f / 1e6 / PEAK_HBM_GBPS, 4)})
    return rows


def cpu_baseline(case, begin, end, hp):
    """The fp64 oracle, as it stands, on the host cores: the gradient of a bounded
    sample of the same chunk (rows of the chunk's span), then AdamW on it."""
    import numpy as np

    from oracle import chunkft_oracle as O
    from paper_2605_21177_amd import workloads as WL

    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = os.cpu_count() or 1
    X64 = WL.as_f64(case.X)
    dY64 = WL.as_f64(case.dY)
    n_in = case.n_in
    # sample: the whole chunk (about 69 GFLOP of fp64 matmul and a 32 Mi-element AdamW)
    sample = end - begin
    b, e = begin, begin + sample
    t0 = time.perf_counter()
    g = O.chunk_wgrad(X64, dY64, b, e, dense=False)
    t1 = time.perf_counter()
    th0 = WL.as_f64(case.W0).reshape(-1)[b:e]
    z = np.zeros(sample)
    O.adamw_step(g, th0, z, z, step=1, **hp)
    t2 = time.perf_counter()
    rows = (e - 1) // n_in - b // n_in + 1
    flops_done = 2.0 * case.T * rows * n_in
    return {
        "value": round(2.0 * case.T * sample / (t1 - t0) / 1e12, 5),
        "unit": "TFLOP/s",
        "cores": int(blas_threads),
        "kind": "oracle",
        "sample": f"the whole chunk, {sample} elements ({rows} rows of fp64 dY^T X via numpy/OpenBLAS, "
                  f"{flops_done / 1e9:.1f} GFLOP in {t1 - t0:.2f} s), then fp64 AdamW on them in {t2 - t1:.2f} s "
                  "(numpy element-wise, 1 thread)",
        "adamw_gbps": round(30.0 * sample / (t2 - t1) / 1e9, 3),
    }


if __name__ == "__main__":
    main()
