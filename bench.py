#!/usr/bin/env python3
"""Benchmark of libtlinattn on one MI355X.

A step is one pass of the whole attention path over one batch of synthetic input:
tlin_layer_attn = history attention over all N rows (split into partitions), causal attention
inside the window, and the merge that joins them.  Inputs are generated on the host from a
seed, uploaded once and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is TFLOP/s of the step (4*B*H*W*N*D history flops plus the
causal half of the window); tokens/s and the fraction of the bf16 MFMA peak are given beside
it.  `roofline` is for the dominant kernel (the history partition kernel), timed with HIP
events on the launch stream inside this run; `cpu_baseline` is the fp64 oracle timed on the
host cores on a bounded sample of the same workload.
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

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_F32_MFMA_TFLOPS = 157.3    # MI355X dense fp32 matrix (the fp32 vector rate is the same figure)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    # after the idle time of the input upload the chip needs some 30-50 ms of load to reach the clocks
    # it then holds: the default warm-up covers that
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed steps run before the warm-up until this much time has passed: the chip needs some "
                         "30-50 ms of the same load to settle at the clocks it then holds (reported as settle_steps)")
    ap.add_argument("--config", type=int, default=4, help="1..4: the fixed workloads (default 4: N=131072, W=512, bf16)")
    ap.add_argument("--combine", choices=("sum", "joint"), default="sum")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--sweep", action="store_true", help="latency-vs-N sweep instead of the single workload")
    ap.add_argument("--workload", choices=("config", "decode", "restore", "slide", "paper", "f32"), default="config",
                    help="config: --config's layer call (default). decode: the cache-hit step of Section 4.2, "
                         "--W newest rows (default 1) query --N history rows (default 131072) through "
                         "tlin_history_attn. restore: the context path's last layer, --N history rows (default "
                         "131072) query --W compressed rows (default 256) through tlin_history_attn. slide: the "
                         "sliding schedule of Section 5.1 over a sequence of --N rows (default 131072) in chunks of "
                         "--W rows (default 512) through tlin_slide_layer_attn. paper: the layer call at the paper's "
                         "own model shape, 12 heads of dimension 36, --W window rows (default 256; 1 = cache-hit "
                         "step through tlin_history_attn) over --N history rows (default 131072). f32: the layer call with fp32 "
                         "inputs, 32 heads of dimension 128, --W window rows (default 512) over --N history rows "
                         "(default 32768)")
    ap.add_argument("--N", type=int, default=None)
    ap.add_argument("--W", type=int, default=None)
    ap.add_argument("--history-only", action="store_true",
                    help="config / f32 / paper workloads: time tlin_history_attn alone instead of the layer call")
    ap.add_argument("--graph", action="store_true",
                    help="also time the steps replayed from a HIP graph (ms_per_step_hip_graph): for the small, launch-bound workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gemm-context", action="store_true",
                    help="skip the context figures measured after the steps (shader clock while stepping; library bf16 "
                         "GEMM for matrix-core-bound workloads; plain read stream for HBM-bound ones)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU work for the oracle sample")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy, so that a rocprofv3 --pmc run of this "
                         "command shows what FETCH_SIZE / WRITE_SIZE read for a kernel of known traffic")
    return ap.parse_args()


def upload(host, dtype, ti, torch, np):
    """Device copies; rows are padded to whole 16-byte pieces when the head dimension is not."""
    dev = {}
    for k, a in host.items():
        t = (torch.from_numpy(a).cuda() if dtype == ti.F32
             else torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16))
        per16 = 16 // t.element_size()
        D = t.shape[-1]
        if D % per16:
            buf = torch.zeros(t.shape[:-1] + ((D + per16 - 1) // per16 * per16,), dtype=t.dtype, device=t.device)
            buf[..., :D] = t
            t = buf[..., :D]
        dev[k] = t
    return dev


def settle(fn, min_ms, torch):
    """Untimed steps until min_ms of wall time have passed (in batches, with a synchronisation after
    each): after the idle time of the input upload the chip ramps its clocks for some tens of
    milliseconds, which a short warm-up would leave inside the timed region.  Returns the number
    of steps run."""
    n = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while min_ms > 0 and (time.perf_counter() - t0) * 1e3 < min_ms:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        n += 10
    return n


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def rotating(Kh, Vh, torch):
    """A history that fits in the 256 MB last-level cache would never be read from HBM again after
    the first step: such workloads rotate through copies of K_hist / V_hist that together exceed
    it.  Returns (next_kv, number of buffer sets)."""
    kv_one = 2 * Kh.numel() * Kh.element_size()
    n_kv = 1 if kv_one >= (512 << 20) else min(16, -(-(512 << 20) // kv_one))

    def copy_of(t):                       # keeps the row padding of tensors whose head dimension needs it
        c = torch.empty_strided(t.shape, t.stride(), dtype=t.dtype, device=t.device)
        c.copy_(t)
        return c

    kv_sets = [(Kh, Vh)] + [(copy_of(Kh), copy_of(Vh)) for _ in range(n_kv - 1)]
    turn = [0]

    def next_kv():
        turn[0] = (turn[0] + 1) % n_kv
        return kv_sets[turn[0]]

    return next_kv, n_kv


def gemm_context(torch, n=8192, iters=50):
    """Context only, never the target: the rate the vendor library's plain bf16 matrix product
    (torch.matmul) sustains on this GPU right after the timed steps.  Under sustained matrix-core load
    the chip clocks well below the 2.4 GHz that the published peak assumes, so this is the practical
    ceiling for a dense contraction on the box the run landed on."""
    try:
        a = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
        b = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
        for _ in range(10):
            a @ b
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(iters):
            a @ b
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t) / iters
        return {"library_bf16_gemm_TFLOPs": 2.0 * n ** 3 / dt / 1e12, "shape": f"{n}x{n}x{n}",
                "kind": "torch.matmul, same GPU, same run"}
    except Exception as e:                   # a context figure must never fail the bench
        return {"library_bf16_gemm_TFLOPs": None, "error": repr(e)}


def read_ceiling(binding, buf, torch, iters=20):
    """Context for HBM-bound workloads, never the peak: the rate at which this GPU feeds a kernel that
    only reads (the library's measurement-aid stream kernel over the history keys, plain and
    non-temporal loads), timed with events on the launch stream."""
    try:
        nbytes = buf.numel() * buf.element_size() if buf.is_contiguous() else 0
        if nbytes < (256 << 20):
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_()
            nbytes = buf.numel()
        st = torch.cuda.current_stream().cuda_stream
        blocks_bytes = 16 * 8 * 256
        read = nbytes // blocks_bytes * blocks_bytes
        out = {"bytes": read, "kind": "libtlinattn stream-read kernel, same GPU, same run"}
        for name, nt in (("plain_loads_GBs", False), ("nontemporal_loads_GBs", True)):
            for _ in range(3):
                binding.profile_stream_read(buf.data_ptr(), nbytes, nt, st)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                binding.profile_stream_read(buf.data_ptr(), nbytes, nt, st)
            e1.record()
            torch.cuda.synchronize()
            out[name] = read / (e0.elapsed_time(e1) / iters * 1e-3) / 1e9
        return out
    except Exception as e:                   # a context figure must never fail the bench
        return {"error": repr(e)}


def sustained_clock(step, torch, seconds=1.2):
    """Context: the shader clock rocm-smi reports while the step runs back to back (the chip is
    power-limited under matrix-core load and settles well below its 2.4 GHz maximum).  None if
    rocm-smi is not available."""
    import re
    import subprocess
    try:
        t_end = time.perf_counter() + seconds
        proc = None
        while time.perf_counter() < t_end or proc is None:
            for _ in range(50):
                step()
            if proc is None and time.perf_counter() > t_end - seconds * 0.6:
                proc = subprocess.Popen(["rocm-smi", "--showclocks"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
            torch.cuda.synchronize()
        text = proc.communicate(timeout=20)[0]
        m = re.search(r"sclk clock level:[^(]*\((\d+)Mhz\)", text)
        return int(m.group(1)) if m else None
    except Exception:
        return None


def cpu_baseline(w, host, target_s, oracle, np, layer=True, joint=False):
    """Oracle on a seeded row sample sized for about target_s seconds; returns the JSON object, the
    sampled rows and the oracle's output for them (which the caller compares with the GPU's).
    layer=True: the layer call (one history softmax plus one window softmax per row, or one joint
    softmax); layer=False: history attention only."""
    def run(rows):
        if layer:
            return oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale,
                                oracle.JOINT if joint else oracle.SUM, rows)
        return oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, rows)[0]
    rng = np.random.default_rng(12345)
    probe = np.sort(rng.choice(w.W, size=min(w.W, 1), replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    run(probe)
    t_probe = time.perf_counter() - t0            # B*H rows in parallel over the cores
    rows_per_head = int(max(1, min(w.W, target_s / max(t_probe, 1e-4) * len(probe))))
    rows = np.sort(rng.choice(w.W, size=rows_per_head, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    ref = run(rows)
    dt = time.perf_counter() - t0
    flops = 4.0 * w.B * w.H * w.D * (len(rows) * w.N + (float(np.sum(rows + 1)) if layer else 0.0))
    return rows, ref, {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{len(rows)} of {w.W} window rows in each of {w.B * w.H} heads, full history, fp64, "
                      f"{dt:.1f} s",
            "window_tokens_per_s": w.B * len(rows) / dt * (1.0),
            "seconds": dt}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every (batch, head) problem is independent; "
              "no multi-GPU path exists). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import tlin_inputs as ti
    import paper_2508_20407_amd as tl
    from paper_2508_20407_amd import binding

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    combine = tl.TLIN_COMBINE_SUM if args.combine == "sum" else tl.TLIN_COMBINE_JOINT

    if args.sweep:
        return sweep(args, ti, tl, binding, torch, np, combine)
    if args.workload == "slide":
        return slide(args, ti, tl, binding, torch, np, combine)

    layer = (args.workload in ("config", "f32") or (args.workload == "paper" and (args.W or 256) > 1)) and not args.history_only
    if args.workload == "config":
        w = ti.config(args.config - 1)
        metric = "history-attention TFLOP/s & tokens/s at N=128K,W=512 bf16; % MFMA peak"
        what = "tlin_layer_attn = history partitions + window causal (one launch) + merge"
    elif args.workload == "paper":
        w = ti.paper_model_point(args.N or 131072, args.W or 256)
        metric = "attention of the paper's own model shape (12 heads x 36), bf16"
        what = ("tlin_layer_attn = history partitions + window causal + merge" if layer else
                "tlin_history_attn = history partitions + merge (cache-hit step)")
    elif args.workload == "f32":
        w = ti.f32_point(args.N or 32768, args.W or 512)
        metric = "layer call with fp32 inputs (fp32 matrix-core products); % fp32 MFMA peak"
        what = "tlin_layer_attn = history partitions + window causal (one launch) + merge"
    elif args.workload == "decode":
        w = ti.decode_point(args.N or 131072, args.W or 1)
        metric = "cache-hit step: newest rows x N-row history, bf16; % HBM peak"
        what = "tlin_history_attn = history partitions + merge"
    else:
        w = ti.restore_point(args.N or 131072, args.W or 256)
        metric = "context-path restoration: N query rows x W_oh compressed rows, bf16"
        what = "tlin_history_attn, one partition"
    if args.history_only:
        what = "tlin_history_attn = history partitions + merge"
    host = ti.make(w) if layer else ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype, ti, torch, np)
    Q, Kh, Vh = dev["Q"], dev["Kh"], dev["Vh"]
    ws = tl.Workspace()

    next_kv, n_kv = rotating(Kh, Vh, torch)

    if layer:
        Kw, Vw = dev["Kw"], dev["Vw"]

        def step():
            k, v = next_kv()
            return tl.tlin_layer_attn(Q, k, v, Kw, Vw, combine=combine, scale=w.scale,
                                      num_splits=args.num_splits, workspace=ws)
    else:
        def step():
            k, v = next_kv()
            return tl.tlin_history_attn(Q, k, v, scale=w.scale, num_splits=args.num_splits, workspace=ws)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    settle_steps = settle(step, args.settle_ms, torch)
    sec = time_steps(step, args.steps, args.warmup, torch)

    # Spread of single steps: the same K steps again, each between its own pair of events on the
    # launch stream (torch's current stream, which the binding passes to the library).
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    step_median, step_min = per_step[len(per_step) // 2], per_step[0]

    # Launch-bound workloads: the same steps replayed from a HIP graph (one graph holds one step per
    # rotated K/V copy), which takes the host's launch path out of the loop.
    graph_ms = None
    if args.graph:
        per_graph = max(n_kv, 1)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(per_graph):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                step()
        replays = max(1, args.steps // per_graph)
        for _ in range(max(1, args.warmup // per_graph)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / (replays * per_graph) * 1e3

    # Per-kernel durations: the same K steps again with event pairs around every launch.
    binding.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms, launches = binding.profile_read()
    binding.profile_enable(False)
    hist_ms = ms[0] / max(launches[0], 1)
    win_ms = ms[1] / max(launches[1], 1)
    merge_ms = ms[2] / max(launches[2], 1)

    flops_h, flops_w = w.flops_history(), (w.flops_window() if layer else 0.0)
    tflops = (flops_h + flops_w) / sec / 1e12
    esz = 4 if w.dtype == ti.F32 else 2
    # Algorithmic bytes of the history kernel: K_hist + V_hist read once; where the query side is
    # the long one (restoration) Q read once and O written once dominate and are counted too.
    kv_bytes = 2.0 * w.B * w.H * w.N * w.D * esz
    if args.workload == "restore":
        kv_bytes += 2.0 * w.B * w.H * w.W * w.D * esz
    # bf16 layer calls run the history partitions and the window blocks in one launch: then that
    # kernel carries the window flops too
    paired = layer and launches[0] > 0 and launches[1] == 0
    hist_tflops = (flops_h + (flops_w if paired else 0.0)) / (hist_ms * 1e-3) / 1e12
    hist_gbs = kv_bytes / (hist_ms * 1e-3) / 1e9
    # Arithmetic intensity of the history kernel is W flop/byte (bf16; W/2 for fp32): it is
    # matrix-core bound when that exceeds the ridge point peak_flops/peak_bw of its operand type
    # (fp32 inputs are multiplied by the fp32 matrix instructions), else HBM bound.
    peak_mfma = PEAK_F32_MFMA_TFLOPS if w.dtype == ti.F32 else PEAK_BF16_MFMA_TFLOPS
    if flops_h / kv_bytes >= peak_mfma * 1e12 / (PEAK_HBM_GBS * 1e9):
        roof = {"bound": "mfma", "achieved": hist_tflops, "peak": peak_mfma, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": hist_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # both fractions, whichever binds (shapes near the ridge sit between the two roofs)
    roof["frac_mfma"] = hist_tflops / peak_mfma
    roof["frac_hbm"] = hist_gbs / PEAK_HBM_GBS
    kname = "attn_f32" if w.dtype == ti.F32 else "attn_bf16"
    # (tlin_history_attn runs calls with few query rows over 1024 or more history rows in its
    # streaming kernel: bf16 at head dimension 128 up to two rows, fp32 up to eight)
    streaming = not layer and w.N >= 1024 and ((w.dtype == ti.BF16 and w.D == 128 and w.W <= 2) or
                                               (w.dtype == ti.F32 and w.W <= 8))
    roof["kernel"] = (f"{kname}_pair_kernel (history partitions + window blocks)" if paired else
                      "decode_kernel (history partitions, streamed through registers)" if streaming else
                      f"{kname}_kernel (history partitions)")
    roof["kernel_ms"] = hist_ms
    roof["traffic"], roof["traffic_source"] = measured_traffic(w.name)

    out = {
        "metric": metric,
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settle_steps, "ms_per_step": sec * 1e3, "ms_per_step_median": step_median, "ms_per_step_min": step_min,
        "ms_per_step_hip_graph": graph_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == ti.F32 else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "D": w.D, "N_history": w.N, "W_window": w.W,
                   "combine": args.combine, "num_splits": binding.num_splits(tl.params_for(Q, w.N, num_splits=args.num_splits)),
                   "step": what, "kv_buffers_rotated": n_kv},
        "window_tokens_per_s": w.B * w.W / sec, "context_tokens_per_s": w.B * w.N / sec,
        "pct_mfma_peak": 100.0 * tflops / peak_mfma,
        "step_GB_per_s": kv_bytes / sec / 1e9, "pct_hbm_peak": 100.0 * kv_bytes / sec / 1e9 / PEAK_HBM_GBS,
        "kernels_ms": {"history": hist_ms, "window_causal": win_ms, "merge": merge_ms},
        "roofline": roof,
    }
    if not args.no_gemm_context:
        # context figures measured on the same GPU in the same run; never used as the peak
        out["context"] = {"sclk_MHz_while_stepping": sustained_clock(step, torch), "sclk_MHz_max": 2400}
        if roof["bound"] == "mfma" and w.dtype != ti.F32:
            out["context"].update(gemm_context(torch))
            if out["context"].get("library_bf16_gemm_TFLOPs"):
                out["context"]["kernel_vs_library_gemm"] = hist_tflops / out["context"]["library_bf16_gemm_TFLOPs"]
        if roof["bound"] == "hbm":
            out["context"]["read_stream"] = read_ceiling(binding, Kh, torch)
            best = out["context"]["read_stream"].get("nontemporal_loads_GBs")
            if best:
                out["context"]["kernel_vs_read_stream"] = hist_gbs / best
    if not args.no_cpu_baseline:
        import oracle
        rows, ref, out["cpu_baseline"] = cpu_baseline(w, host, args.cpu_seconds, oracle, np, layer, args.combine == "joint")
        # the output of the timed call against the oracle rows just computed (every K/V copy that
        # the steps rotate through holds the same values)
        got = step()[:, :, torch.from_numpy(rows).long().cuda()].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        out["parity"] = {"rows": int(len(rows) * w.B * w.H), "rows_per_head": int(len(rows)), "max_abs": float(err.max()),
                         "mean_abs": float(err.mean()), "against": "the oracle rows of cpu_baseline"}
        if w.dtype == ti.F32:
            rms = float(np.sqrt(np.mean(ref * ref)))
            out["parity"]["max_rel"] = float(np.max(err / np.maximum(np.abs(ref), rms)))     # denominator floored at the rms
            big = np.abs(ref) > rms
            out["parity"]["max_rel_unfloored_above_rms"] = float(np.max(err[big] / np.abs(ref[big]))) if big.any() else None
            out["parity"]["ok"] = out["parity"]["max_rel"] <= 1e-5
        else:
            out["parity"]["ok"] = bool(err.max() <= 2e-2 and err.mean() <= 5e-3)
    print(json.dumps(out), flush=True)
    if "parity" in out and not out["parity"]["ok"]:
        print("bench.py: the timed call's output is outside the tolerance against the oracle", file=sys.stderr)
        sys.exit(1)


# HBM bytes per launch of the dominant kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (two runs of this script with --calibrate-copy; raw readings, commands and the scale factors of the
# two counters are in the profile files named here).  A figure is only reported while the kernel
# sources are the ones it was measured on (csrc_sha16 below = kernel_sources_sha16() at that time);
# otherwise `traffic` is null and `traffic_source` says why.
_SHA = "6958dfe247894b72"      # kernel_sources_sha16() when the counters below were read
MEASURED_TRAFFIC = {
    # workload: (FETCH_SIZE KiB x 2.0 + WRITE_SIZE KiB x 1.0) x 1024, profile file with the raw readings
    "cfg4_bf16_N131072_W512": {"bytes": int(1_056_966.8 * 2.0 * 1024) + int(41_600.0 * 1024),   # 2.016 GiB fetched + 40.6 MiB written
                               "profile": "profiles/attn_bf16_pair_cfg4_pmc.md", "csrc_sha16": _SHA},
    "decode_bf16_N131072_W1": {"bytes": int(1_055_860.0 * 2.0 * 1024) + int(576.2 * 1024),      # 2.014 GiB fetched + 0.6 MiB written
                               "profile": "profiles/decode_bf16_w1.md", "csrc_sha16": _SHA},
    "cfg3_bf16_N32768_W256_peaky": {"bytes": int(532_236.9 * 2.0 * 1024) + int(41_600.0 * 1024),    # 1.015 GiB + 40.6 MiB
                                    "profile": "profiles/attn_bf16_pair_cfg3_kernel_trace.md", "csrc_sha16": _SHA},
    "restore_bf16_Q131072_K256": {"bytes": int(526_450.8 * 2.0 * 1024) + int(1_048_576.0 * 1024),    # 1.004 GiB (Q) + 1 GiB (O)
                                  "profile": "profiles/attn_bf16_resident_restore_kernel_trace.md", "csrc_sha16": _SHA},
    "f32_N131072_W1": {"bytes": int(2_108_624.1 * 2.0 * 1024) + int(576.3 * 1024),                  # 4.022 GiB + 0.6 MiB
                       "profile": "profiles/decode_f32_w1.md", "csrc_sha16": _SHA},
    "f32_N32768_W512": {"bytes": int(540_852.3 * 2.0 * 1024) + int(41_600.0 * 1024),                # 1.032 GiB + 40.6 MiB
                        "profile": "profiles/attn_f32_pair_N32768_W512.md", "csrc_sha16": _SHA},
    "paper_bf16_H12_D36_N999754_W256": {"bytes": int(955_056.1 * 2.0 * 1024) + int(26_136.0 * 1024),   # 1.822 GiB + 25.5 MiB
                                        "profile": "profiles/attn_bf16_pair_paper_hd36_N999754.md", "csrc_sha16": _SHA},
}


def kernel_sources_sha16():
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2508_20407_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(name):
    m = MEASURED_TRAFFIC.get(name)
    now = kernel_sources_sha16()
    if m is None:
        return None, {"note": "not measured for this workload", "csrc_sha16": now}
    if m["csrc_sha16"] != now:
        return None, {"note": "kernel sources changed since the counter run in " + m["profile"], "csrc_sha16": now,
                      "measured_at_csrc_sha16": m["csrc_sha16"]}
    return m["bytes"], {"profile": m["profile"], "csrc_sha16": now}


def slide(args, ti, tl, binding, torch, np, combine):
    """One call of tlin_slide_layer_attn over a whole sequence: every chunk of W rows against all
    earlier chunks plus causal attention inside the chunk."""
    L, W = args.N or 131072, args.W or 512
    w = ti.Workload(f"slide_bf16_L{L}_W{W}", 1, 32, 128, L, W, ti.BF16, 1.0, 204077)
    shape = (w.B, w.H, L, w.D)
    host = {name: ti.normal(shape, w.dtype, w.seed, tag, w.mul) for name, tag in
            (("Q", ti.TAG_Q), ("Kh", ti.TAG_KH), ("Vh", ti.TAG_VH), ("Kw", ti.TAG_KW), ("Vw", ti.TAG_VW))}
    dev = upload(host, w.dtype, ti, torch, np)
    ws = tl.Workspace()

    def step():
        return tl.tlin_slide_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], W, combine=combine,
                                        scale=w.scale, num_splits=args.num_splits, workspace=ws)

    settle_steps = settle(step, args.settle_ms, torch)
    sec = time_steps(step, args.steps, args.warmup, torch)
    binding.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms, launches = binding.profile_read()
    binding.profile_enable(False)
    hist_ms, win_ms, merge_ms = (ms[i] / max(launches[i], 1) for i in range(3))
    starts = np.arange(0, L, W, dtype=np.float64)
    lens = np.minimum(W, L - starts)
    bh = w.B * w.H
    flops_h = 4.0 * bh * w.D * float(np.sum(lens * starts))
    flops_w = 4.0 * bh * w.D * float(np.sum(lens * (lens + 1) / 2))
    kv_bytes = 2.0 * bh * w.D * 2 * float(np.sum(starts))          # every chunk reads its history once
    tflops = (flops_h + flops_w) / sec / 1e12
    hist_tflops = flops_h / (hist_ms * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": hist_tflops, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": hist_tflops / PEAK_BF16_MFMA_TFLOPS, "kernel": "attn_bf16_kernel (chunk histories)",
            "kernel_ms": hist_ms, "traffic": None}
    if W < PEAK_BF16_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        gbs = kv_bytes / (hist_ms * 1e-3) / 1e9
        roof.update({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS})
    out = {"metric": "sliding schedule over a whole sequence (Section 5.1), bf16: TFLOP/s and tokens/s",
           "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "settle_steps": settle_steps, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": w.name, "B": w.B, "H": w.H, "D": w.D, "L_sequence": L, "W_chunk": W,
                      "combine": args.combine, "step": "tlin_slide_layer_attn = chunk histories + chunk causal + merge"},
           "tokens_per_s": w.B * L / sec, "pct_mfma_peak": 100.0 * tflops / PEAK_BF16_MFMA_TFLOPS,
           "kernels_ms": {"history": hist_ms, "window_causal": win_ms, "merge": merge_ms}, "roofline": roof}
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(12345)
        probe = np.sort(rng.choice(L, size=2, replace=False)).astype(np.int32)
        t0 = time.perf_counter()
        oracle.slide(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, W,
                     oracle.JOINT if args.combine == "joint" else oracle.SUM, probe)
        t_probe = time.perf_counter() - t0
        n = int(max(2, min(L, args.cpu_seconds / max(t_probe, 1e-4) * len(probe))))
        rows = np.sort(rng.choice(L, size=n, replace=False)).astype(np.int32)
        t0 = time.perf_counter()
        ref = oracle.slide(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, W,
                           oracle.JOINT if args.combine == "joint" else oracle.SUM, rows)
        dt = time.perf_counter() - t0
        got = step()[:, :, torch.from_numpy(rows).long().cuda()].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        out["parity"] = {"rows": int(n * bh), "rows_per_head": int(n), "max_abs": float(err.max()), "mean_abs": float(err.mean()),
                         "ok": bool(err.max() <= 2e-2 and err.mean() <= 5e-3), "against": "the oracle rows of cpu_baseline"}
        keys = float(np.sum(rows + 1))                # history rows + visible window rows of each sampled position
        out["cpu_baseline"] = {"value": 4.0 * bh * w.D * keys / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(),
                               "kind": "oracle", "sample": f"{n} of {L} sequence positions in each of {bh} heads, fp64, "
                                                           f"{dt:.1f} s", "seconds": dt}
    print(json.dumps(out), flush=True)


def sweep(args, ti, tl, binding, torch, np, combine):
    """Latency of tlin_history_attn vs N at fixed W, with a least-squares line per W (the cost
    model of Section 4.1 predicts exact linearity in N)."""
    pts = ti.sweep_points()
    ws = tl.Workspace()
    results = []
    for w in pts:
        host = ti.make(w, which=("Q", "Kh", "Vh"))
        dev = upload(host, w.dtype, ti, torch, np)
        Q, Kh, Vh = dev["Q"], dev["Kh"], dev["Vh"]
        next_kv, n_kv = rotating(Kh, Vh, torch)
        sec = time_steps(lambda: tl.tlin_history_attn(Q, *next_kv(), scale=w.scale, workspace=ws), args.steps, args.warmup, torch)
        tf = w.flops_history() / sec / 1e12
        gbs = 2.0 * w.B * w.H * w.N * w.D * 2 / sec / 1e9
        results.append({"N": w.N, "W": w.W, "kv_buffers_rotated": n_kv, "ms": sec * 1e3, "TFLOP/s": tf, "GB/s": gbs,
                        "pct_mfma_peak": 100 * tf / PEAK_BF16_MFMA_TFLOPS, "pct_hbm_peak": 100 * gbs / PEAK_HBM_GBS})
        print(json.dumps(results[-1]), file=sys.stderr, flush=True)
        del dev, Q, Kh, Vh, host, next_kv
        torch.cuda.empty_cache()
    fits = {}
    for W in sorted({r["W"] for r in results}):
        xs = np.array([r["N"] for r in results if r["W"] == W], dtype=np.float64)
        ys = np.array([r["ms"] for r in results if r["W"] == W], dtype=np.float64)
        a, b = np.polyfit(xs, ys, 1)
        pred = a * xs + b
        r2 = 1.0 - float(((ys - pred) ** 2).sum() / ((ys - ys.mean()) ** 2).sum())
        fits[str(W)] = {"ms_per_history_row": a, "intercept_ms": b, "r2": r2}
    wd = ti.degenerate_causal()
    host = ti.make(wd, which=("Q", "Kw", "Vw"))
    dev = upload(host, wd.dtype, ti, torch, np)
    sec = time_steps(lambda: tl.tlin_layer_attn(dev["Q"], None, None, dev["Kw"], dev["Vw"], combine=combine, scale=wd.scale),
                     args.steps, args.warmup, torch)
    degenerate = {"N": 0, "W": wd.W, "ms": sec * 1e3, "TFLOP/s": wd.flops_window() / sec / 1e12}
    print(json.dumps({"metric": "latency vs N sweep (tlin_history_attn, bf16, B=1, H=32, D=128)", "points": results,
                      "linear_fit": fits, "empty_history_causal": degenerate, "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "data": "synthetic"}), flush=True)


if __name__ == "__main__":
    main()
