#!/usr/bin/env python3
"""Benchmark of the NanoQuant binary low-rank forward on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--workload cfg2|cfg3|cfg4] [--batch B]

One "step" is one pass of the whole hot path (input quantisation, stage 1
t = V^T (s_in . x), quantisation of t, stage 2 y = s_out . (U t)) over every layer of
the workload, issued as ONE nq_plan_forward: four kernel launches, or two when the stage
kernels quantise their own input (batch 1, reductions of at most 1024 / 4096 elements -- the
default workload).

Default workload "cfg2": the Llama-2-7B-shaped attention projection 4096x4096, r = 1024
(0.5 bit/weight), bf16 activations, decode batch 1 -- as a pool of distinct seeded layer
instances whose packed weights (1.09 GB) are four times the 256 MB Infinity Cache, so every
step streams its bits from HBM rather than from cache.  All inputs are resident in HBM
before the timed region.

Prints ONE JSON line.  `value` is effective weight GB/s = bytes of the stored
factorization (r(n+m)/8 + 2(n+m) per layer, Appendix F.5) read per second.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16/bf16 MFMA rate


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4"])
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--pool", type=int, default=1024, help="cfg2: number of distinct layer instances")
    ap.add_argument("--layers", type=int, default=0, help="cfg3/cfg4: decoder layers (0 = all)")
    ap.add_argument("--y-dtype", default="f32", choices=["f32", "bf16", "f16"],
                    help="output type of the layers (f32 is the parity-checked default of the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target oracle time for the cpu_baseline sample")
    ap.add_argument("--quick", action="store_true",
                    help="headline workload only: skip the extra fields (70B stack decode, config-5 prefill)")
    ap.add_argument("--case", default="",
                    help="run ONE of the side workloads only and print its JSON (for profiling a single case): "
                         "prefill:<gate|down>:<batch> | pool_b<1..8>[:two_slice] | stack3 | stack4 | chain3 | chain4 | transposed | admm")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference for rocprofv3 --pmc byte counters)")
    return ap.parse_args()


def build_workload(args):
    """Returns list of (shape, LayerData, x_numpy) for the chosen workload."""
    from paper_2602_06694_amd import synth
    out = []
    if args.workload == "cfg2":
        shp = synth.CONFIGS[2].block[0]
        for i in range(args.pool):
            out.append((shp, synth.gen_layer(2, i, 0, shp), synth.gen_layer_x(2, i, 0, shp, args.batch, "bf16")))
        name = f"cfg2: {args.pool} x [4096x4096 r=1024], decode batch {args.batch}, bf16 x"
    else:
        cfg = 3 if args.workload == "cfg3" else 4
        c = synth.CONFIGS[cfg]
        nl = args.layers or c.n_layers
        for layer, li, shp in synth.iter_config_layers(cfg, nl):
            out.append((shp, synth.gen_layer(cfg, layer, li, shp), synth.gen_layer_x(cfg, layer, li, shp, args.batch, "bf16")))
        name = f"cfg{cfg}: {c.name} ({nl} layers x 7 linears), decode batch {args.batch}, bf16 x"
    return name, out


def prewarm(run, seconds=0.05):
    """The chip changes its power state a few milliseconds into a sustained load, which stalls the
    queue for about a millisecond once; run `run` untimed until that is over (then come the W
    warm-up steps of the contract)."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            run()
        torch.cuda.synchronize()


def timed_windows(run, steps, windows=5):
    """Times `windows` back-to-back windows of `steps` calls of run() (wall clock around a device
    synchronisation each); returns per-step milliseconds of every window."""
    import torch
    out = []
    for _ in range(windows):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) * 1e3 / steps)
    return out


def window_stats(ms):
    s = sorted(ms)
    return {"median": s[len(s) // 2], "min": s[0], "max": s[-1], "windows": len(s)}


class ClockSampler:
    """Observed engine / memory clocks while a load runs: rocm-smi is started in the background just
    before a timed region and read afterwards (clocks are left at their defaults)."""

    def __init__(self):
        import shutil
        import subprocess
        self.proc = None
        exe = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
        # under a profiler every child process is itself instrumented (and initialises the GPU before it can start
        # another program): no side process is started then, and the clocks are reported as null
        if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
            return
        try:
            self.proc = subprocess.Popen(["bash", "-c", f"sleep 0.3; {exe} --showclocks"], stdout=subprocess.PIPE,
                                         stderr=subprocess.DEVNULL, text=True)
        except OSError:
            self.proc = None

    def read(self):
        import re
        if self.proc is None:
            return None
        try:
            text = self.proc.communicate(timeout=20)[0]
        except Exception:
            return None
        out = {}
        for name in ("sclk", "mclk", "fclk"):
            m = re.search(rf"{name} clock level: \d+: \((\d+)Mhz\)", text)
            if m:
                out[name + "_MHz"] = int(m.group(1))
        return out or None


def algorithmic_bytes(shp, batch, y_size=4):
    """Bytes the method itself must move for one forward of one layer."""
    bits = shp.r * (shp.d_in + shp.d_out) // 8
    scales = 2 * (shp.d_in + shp.d_out)
    x = batch * shp.d_in * 2
    y = batch * shp.d_out * y_size
    t = 2 * batch * shp.r * 4      # intermediate written by stage 1 and read back for stage 2
    return bits + scales, bits + scales + x + y + t


def stage_bytes(shp, batch, y_size=4, self_quantising=(False, False)):
    """Algorithmic bytes of the two streaming launches for one layer:
    stage 1 reads the V bits and the 3-byte fixed-point x', writes t (fp32);
    stage 2 reads the U bits, the 3-byte fixed-point t and s_out (fp16), writes y (y_size bytes each).
    A stage that quantises its own input reads that input as it is instead (bf16 x and fp16 s_in;
    fp32 t)."""
    in1 = (2 * batch * shp.d_in + 2 * shp.d_in) if self_quantising[0] else 3 * batch * shp.d_in
    in2 = 4 * batch * shp.r if self_quantising[1] else 3 * batch * shp.r
    s1 = shp.d_in * shp.r // 8 + in1 + 4 * batch * shp.r
    s2 = shp.d_out * shp.r // 8 + 2 * shp.d_out + in2 + y_size * batch * shp.d_out
    return s1, s2


SCHEDULE_KERNEL = {1: "nq::stage_stream_kernel", 4: "nq::stage_split_kernel<W=4>", 16: "nq::stage_split_kernel<W=16>",
                   8: "nq::stage_shared_kernel", 9: "nq::stage_shared_kernel<resident input>",
                   10: "nq::stage_shared_kernel<two slices>", 11: "nq::stage_shared_kernel<resident input, two slices>", 32: "nq::stage_fused_kernel", 33: "nq::stage_selfq_kernel<W=1>",
                   34: "nq::stage_selfq_kernel<W=4>"}


def cpu_baseline(work, batch, target_s):
    """Oracle (Tier B, fp64, OpenMP over the host cores) on a bounded sample of the same layers:
    it walks the workload's layers in order (wrapping around) until about `target_s` seconds are spent."""
    import oracle
    from paper_2602_06694_amd import synth
    wbytes, n, used = 0, 0, 1
    t0 = time.perf_counter()
    while True:
        shp, data, x = work[n % len(work)]
        _, used = oracle.forward_factored(data.U_words, data.V_words, data.s_out, data.s_in, shp.d_out, shp.d_in,
                                          shp.r, synth.x_as_f64(x, "bf16"), threads=0, return_threads=True)
        wbytes += algorithmic_bytes(shp, batch)[0]
        n += 1
        dt = time.perf_counter() - t0
        if dt >= target_s:
            break
    # the same oracle on one thread, on a few layers (about a fifth of the time again)
    t1 = time.perf_counter()
    wb1, n1 = 0, 0
    while True:
        shp, data, x = work[n1 % len(work)]
        oracle.forward_factored(data.U_words, data.V_words, data.s_out, data.s_in, shp.d_out, shp.d_in, shp.r,
                                synth.x_as_f64(x, "bf16"), threads=1)
        wb1 += algorithmic_bytes(shp, batch)[0]
        n1 += 1
        dt1 = time.perf_counter() - t1
        if dt1 >= target_s / 5:
            break
    return {"value": wbytes / dt / 1e9, "unit": "GB/s", "cores": int(used), "kind": "oracle",
            "sample": f"{n} layer forwards (the workload's layers in order, wrapping), fp64 factored oracle, {dt:.1f} s",
            "layers_per_s": n / dt,
            "single_thread": {"value": wb1 / dt1 / 1e9, "unit": "GB/s", "cores": 1,
                              "sample": f"{n1} layer forwards, {dt1:.1f} s"}}


def measured_traffic(workload_name, stage, kernel_name):
    """HBM bytes per launch of the given stage from the committed rocprofv3 --pmc summary of this
    workload (FETCH_SIZE + WRITE_SIZE, each scaled by the copy-kernel calibration), or None if the
    summary does not cover it: another workload, or a stage that ran a different kernel then (the
    summary's line for the stage must name the kernel this run launched, e.g. nq::stage_selfq_kernel<4)."""
    path = os.path.join(ROOT, "profiles", "stage_kernels_cfg2_pool_pmc.txt")
    # "nq::stage_selfq_kernel<W=4>" -> "nq::stage_selfq_kernel<4"
    key = kernel_name.replace("<W=", "<").rstrip(">").split(" ")[0]
    try:
        text = open(path).read()
        want, same_kernel, value = None, False, None
        for line in text.splitlines():
            if line.startswith("workload:"):
                want = line.split(":", 1)[1].strip()
            if f"[{stage}:" in line and line.startswith(key):
                same_kernel = True
            if line.startswith(f"traffic_bytes_per_launch_{stage}:") and want == workload_name:
                value = float(line.split(":", 1)[1])
        return value if same_kernel else None
    except OSError:
        pass
    return None


def graph_replay_ms(run, steps, windows=3):
    """`run` captured once into a HIP graph (torch's capture stream), then replayed: median ms per replay,
    or the reason the capture failed -- reported, not hidden."""
    import torch
    try:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):                    # first calls outside the capture (lazy set-up)
            run()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        prewarm(graph.replay, 0.02)
        ms = window_stats(timed_windows(graph.replay, steps, windows))["median"]
        del graph
        return ms
    except Exception as e:
        return f"capture failed: {e}"


def time_stack(cfg, batch, steps=10, warmup=2):
    """Whole decoder stack of config 3 / 4 as one plan of independent layers: step time (median of five
    windows), weight GB/s and per-kernel roofline; and the same stack as a loop of single-layer calls."""
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    handles, xs, ys, wbytes, abytes, sb1, sb2 = [], [], [], 0, 0, 0, 0
    for layer, li, shp in synth.iter_config_layers(cfg):
        data = synth.gen_layer(cfg, layer, li, shp)
        handles.append(nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out,
                                          data.s_in, nq.NQ_BF16))
        x = synth.gen_layer_x(cfg, layer, li, shp, batch, "bf16")
        xs.append(torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda())
        ys.append(torch.empty((batch, shp.d_out), dtype=torch.float32, device="cuda"))
        wb, ab = algorithmic_bytes(shp, batch)
        wbytes += wb
        abytes += ab
        sb1 += stage_bytes(shp, batch)[0]
        sb2 += stage_bytes(shp, batch)[1]
    plan = nq.nq_plan_create(handles, xs, ys, batch)
    prewarm(lambda: nq.nq_plan_forward(plan))
    for _ in range(warmup):
        nq.nq_plan_forward(plan)
    win = timed_windows(lambda: nq.nq_plan_forward(plan), steps)
    ms = window_stats(win)["median"]
    pk = np.zeros(4)
    for _ in range(5):
        pk += np.array(nq.nq_plan_forward_timed(plan))
    pk /= 5
    # the same stack as a plain loop of single-layer calls (two to four launches per layer on one stream)
    def loop():
        for h, x, y in zip(handles, xs, ys):
            nq.nq_binlr_forward(h, x, y, batch)
    prewarm(loop, 0.02)
    ms_loop = window_stats(timed_windows(loop, 2, 3))["median"]
    ms_loop_graph = graph_replay_ms(loop, 2)
    ms_plan_graph = graph_replay_ms(lambda: nq.nq_plan_forward(plan), steps)
    res = {"layers": len(handles), "ms_per_step": ms, "ms_per_step_windows": window_stats(win),
           "weight_GBps": wbytes / ms / 1e6, "tokens_per_s": batch / (ms * 1e-3),
           "ms_per_step_loop_of_single_calls": ms_loop, "ms_per_step_hip_graph_of_that_loop": ms_loop_graph,
           "ms_per_step_hip_graph_of_the_plan": ms_plan_graph,
           "kernel_ms": {"quantize_x": pk[0], "stage1": pk[1], "quantize_t": pk[2], "stage2": pk[3]},
           "stage1_GBps": sb1 / pk[1] / 1e6, "stage2_GBps": sb2 / pk[3] / 1e6,
           "stage1_frac_of_hbm_peak": sb1 / pk[1] / 1e6 / HBM_PEAK_GBPS,
           "stage2_frac_of_hbm_peak": sb2 / pk[3] / 1e6 / HBM_PEAK_GBPS}
    nq.nq_plan_destroy(plan)
    for h in handles:
        nq.nq_binlr_destroy(h)
    return res


def time_stack_in_dependency_order(cfg, steps=10):
    """The stack of config 3 / 4 at batch 1 with every layer reading the output of the layer before it
    (q -> o -> gate -> down -> the next block's q, k, v; k, v and up are computed as well): each of the
    2 x 4 x blocks stages waits for all of the one before.  Scales are multiplied by powers of two so that
    the chain keeps a magnitude near one (synth.gen_chained_stack).  Three ways to run it: the executor
    (one persistent launch per token), four plans per block back to back on the stream, single calls."""
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    c = synth.CONFIGS[cfg]
    layers = synth.gen_chained_stack(cfg)
    n = len(layers)
    level, src = synth.chain_spec(n // 7)
    hs, ys, wbytes = [], [], 0
    for i, d in enumerate(layers):
        shp = d.shape
        hs.append(nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, d.U_words, d.V_words, d.s_out, d.s_in,
                                     nq.NQ_BF16 if src[i] < 0 else nq.NQ_F32))
        ys.append(torch.zeros((1, shp.d_out), dtype=torch.float32, device="cuda"))
        wbytes += algorithmic_bytes(shp, 1)[0]
    x0n = synth.gen_x(1, c.block[0].d_in, synth.seed_for(cfg, 0, 0, synth.T_X), "bf16")
    x0 = torch.from_numpy(x0n.view(np.int16).copy()).view(torch.bfloat16).cuda()
    xs = [x0 if s < 0 else ys[s] for s in src]

    def single():
        for h, x, y in zip(hs, xs, ys):
            nq.nq_binlr_forward(h, x, y, 1)
    single()
    torch.cuda.synchronize()
    ref = [y.clone() for y in ys]
    ex = nq.nq_exec_create(hs, xs, ys, level)
    for y in ys:
        y.zero_()
    nq.nq_exec_forward(ex)
    nq.nq_exec_status(ex)
    identical = all(torch.equal(a, b) for a, b in zip(ys, ref))
    prewarm(lambda: nq.nq_exec_forward(ex))
    win = timed_windows(lambda: nq.nq_exec_forward(ex), steps)
    nq.nq_exec_status(ex)
    ms = window_stats(win)["median"]
    n_wg, n_tasks, lds = nq.nq_exec_info(ex)
    # four plans per block (q, k, v | o | gate, up | down), each two launches, back to back on the stream
    plans = []
    for base in range(0, n, 7):
        for group in ((0, 1, 2), (3,), (4, 5), (6,)):
            idx = [base + g for g in group]
            plans.append(nq.nq_plan_create([hs[i] for i in idx], [xs[i] for i in idx], [ys[i] for i in idx], 1))

    def levels():
        for lp in plans:
            nq.nq_plan_forward(lp)
    prewarm(levels, 0.02)
    ms_levels = window_stats(timed_windows(levels, 3, 3))["median"]
    ms_single = window_stats(timed_windows(single, 2, 3))["median"]
    ms_levels_graph = graph_replay_ms(levels, 3)
    ms_exec_graph = graph_replay_ms(lambda: nq.nq_exec_forward(ex), steps)
    nq.nq_exec_status(ex)
    for lp in plans:
        nq.nq_plan_destroy(lp)
    nq.nq_exec_destroy(ex)
    for h in hs:
        nq.nq_binlr_destroy(h)
    phases = 2 * (level[-1] + 1)
    return {"layers": n, "dependent_stages": phases, "executor_ms_per_step": ms, "executor_windows": window_stats(win),
            "executor_us_per_stage": ms * 1e3 / phases, "executor_weight_GBps": wbytes / ms / 1e6,
            "executor_bit_identical_to_single_calls": bool(identical),
            "executor_workgroups": n_wg, "executor_tasks": n_tasks, "executor_lds_bytes": lds,
            "four_plans_per_block_ms_per_step": ms_levels, "single_calls_ms_per_step": ms_single,
            "hip_graph_of_the_four_plans_per_block_ms_per_step": ms_levels_graph,
            "hip_graph_of_the_executor_launch_ms_per_step": ms_exec_graph}


def time_pool_batch(pool, batch, steps=10, warmup=2, two_slice=False):
    """Config 2's layer at a decode batch other than the headline's (the metric is quoted at batch 8 too):
    the same rotating pool of distinct instances, one plan.  two_slice: with the option that feeds the launches of
    batch 6..8 16-bit fixed point (NOT the exact path: about 3e-4 of the largest output instead of 1.5e-6)."""
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    if two_slice:
        nq.nq_set_option("two_slice_b8", 1)
    shp = synth.CONFIGS[2].block[0]
    handles, xs, ys = [], [], []
    for i in range(pool):
        data = synth.gen_layer(2, i, 0, shp)
        handles.append(nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out,
                                          data.s_in, nq.NQ_BF16))
        x = synth.gen_layer_x(2, i, 0, shp, batch, "bf16")
        xs.append(torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda())
        ys.append(torch.empty((batch, shp.d_out), dtype=torch.float32, device="cuda"))
    plan = nq.nq_plan_create(handles, xs, ys, batch)
    if two_slice:
        nq.nq_set_option("two_slice_b8", None)        # a plan keeps the schedules of its creation
    prewarm(lambda: nq.nq_plan_forward(plan))
    for _ in range(warmup):
        nq.nq_plan_forward(plan)
    win = timed_windows(lambda: nq.nq_plan_forward(plan), steps)
    ms = window_stats(win)["median"]
    pk = np.zeros(4)
    for _ in range(5):
        pk += np.array(nq.nq_plan_forward_timed(plan))
    pk /= 5
    wb, ab = algorithmic_bytes(shp, batch)
    s1, s2 = stage_bytes(shp, batch)
    res = {"layers": pool, "batch": batch, "ms_per_step": ms, "ms_per_step_windows": window_stats(win),
           "schedules": nq.nq_plan_schedules(plan), "weight_GBps": pool * wb / ms / 1e6,
           "algorithmic_GBps": pool * ab / ms / 1e6, "tokens_per_s_per_layer": batch * pool / (ms * 1e-3),
           "kernel_ms": {"quantize_x": pk[0], "stage1": pk[1], "quantize_t": pk[2], "stage2": pk[3]},
           "stage1_GBps": pool * s1 / pk[1] / 1e6, "stage2_GBps": pool * s2 / pk[3] / 1e6}
    nq.nq_plan_destroy(plan)
    for h in handles:
        nq.nq_binlr_destroy(h)
    return res


def time_single_layer(cfg, reps=200):
    """One layer through nq_binlr_forward, back to back (weights stay in cache): launch-bound latency."""
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    c = synth.CONFIGS[cfg]
    shp = c.block[0]
    data = synth.gen_layer(cfg, 0, 0, shp)
    h = nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out, data.s_in,
                           nq.DTYPE_BY_NAME[c.x_dtype])
    xb = synth.gen_layer_x(cfg, 0, 0, shp, 1, c.x_dtype)
    x = torch.from_numpy(xb.view(np.int16).copy()).view(torch.bfloat16).cuda() if c.x_dtype == "bf16" \
        else torch.from_numpy(np.ascontiguousarray(xb)).cuda()
    y = torch.empty((1, shp.d_out), dtype=torch.float32, device="cuda")
    prewarm(lambda: nq.nq_binlr_forward(h, x, y, 1), 0.02)
    for _ in range(20):
        nq.nq_binlr_forward(h, x, y, 1)
    win = timed_windows(lambda: nq.nq_binlr_forward(h, x, y, 1), reps)
    us = window_stats(win)["median"] * 1e3
    wb, _ = algorithmic_bytes(shp, 1)
    nq.nq_binlr_destroy(h)
    return {"shape": [shp.d_out, shp.d_in, shp.r], "us_per_forward": us, "cache_hot_weight_GBps": wb / us / 1e3}


def time_transposed():
    """The transposed product w = V (U^T (s_out . g)) from the resident tiles against the forward without output scale,
    on config 2's layer and on config 5's down layer, batch 1 / 8 / 64 (microseconds per call)."""
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    res = {}
    for cfg, li in ((2, 0), (5, 1)):
        shp = synth.CONFIGS[cfg].block[li]
        data = synth.gen_layer(cfg, 0, li, shp)
        h = nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out, data.s_in, nq.NQ_BF16)
        for batch in (1, 8, 64):
            g = torch.randn((batch, shp.d_out), dtype=torch.float32, device="cuda")
            w = torch.empty((batch, shp.d_in), dtype=torch.float32, device="cuda")
            x = torch.randn((batch, shp.d_in), dtype=torch.float32, device="cuda").to(torch.bfloat16)
            z = torch.empty((batch, shp.d_out), dtype=torch.float32, device="cuda")
            out = {}
            for name, f in (("transposed_us", lambda: nq.nq_binlr_forward_transposed_unscaled(h, g, w, batch)),
                            ("forward_unscaled_us", lambda: nq.nq_binlr_forward_unscaled(h, x, z, batch))):
                prewarm(f, 0.02)
                win = timed_windows(f, 20, 5)
                out[name] = window_stats(win)["median"] * 1e3
            res[f"{shp.name}_{shp.d_out}x{shp.d_in}_r{shp.r}_B{batch}"] = out
        nq.nq_binlr_destroy(h)
    return res


def time_lb_admm(n=4096, m=4096, r=1024, iters=10, power_iters=8, with_oracle=False):
    """LB-ADMM (Section 3.2 Step 2-2) on one synthetic matrix of config 2's shape: time per iteration, the
    binary64 GEMM behind it on the iteration's three product shapes, and (optionally) one oracle iteration."""
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=42)
    dev = lambda a: torch.from_numpy(a).cuda()
    dw, du0, dv0 = dev(w), dev(u0), dev(v0)
    nbytes = nq.nq_lb_admm_workspace_bytes(n, m, r)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = [torch.empty((n if i % 2 == 0 else m, r), dtype=torch.float64, device="cuda") for i in range(6)]

    def run(k):
        nq.nq_lb_admm(dw, n, m, r, du0, dv0, k, 1.0, 20.0, 1e-3, power_iters, out[0], out[1], out[2], out[3], out[4], out[5], ws, nbytes)
    run(2)
    torch.cuda.synchronize()
    win = []
    for _ in range(5):
        t0 = time.perf_counter(); run(0); torch.cuda.synchronize(); t_init = time.perf_counter() - t0
        t0 = time.perf_counter(); run(iters); torch.cuda.synchronize(); t_all = time.perf_counter() - t0
        win.append((t_all - t_init) * 1e3 / iters)
    ms = window_stats(win)["median"]
    # algorithmic flops of one iteration: two products with W, two symmetric Gram matrices, two Cholesky
    # factorisations, and two triangular solves for every row of U and of V
    flops = 2 * (2.0 * n * m * r) + (m + n) * float(r) * r + 2 * r ** 3 / 3.0 + 2.0 * (n + m) * r * r
    res = {"shape": [n, m, r], "iterations_timed": iters, "power_iters": power_iters, "ms_per_iteration": ms,
           "ms_per_iteration_windows": window_stats(win), "algorithmic_GFLOP_per_iteration": flops / 1e9,
           "TFLOPs_algorithmic": flops / ms / 1e9, "frac_of_fp64_matrix_peak": flops / ms / 1e9 / 78.6, "dgemm": {}}
    for name, ta, tb, M, N, K in (("W.V", 0, 0, n, r, m), ("W^T.U", 1, 0, m, r, n), ("V^T.V", 1, 0, r, r, m), ("RHS.Hinv", 0, 0, n, r, r),
                                  ("4096^3", 0, 0, 4096, 4096, 4096)):
        a = torch.randn((K, M) if ta else (M, K), dtype=torch.float64, device="cuda")
        b = torch.randn((K, N), dtype=torch.float64, device="cuda")
        c = torch.empty((M, N), dtype=torch.float64, device="cuda")
        f = lambda: nq.nq_dgemm(ta, tb, M, N, K, 1.0, a, a.shape[1], b, N, 0.0, c, N)
        prewarm(f, 0.03)
        gw = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                f()
            e1.record()
            torch.cuda.synchronize()
            gw.append(e0.elapsed_time(e1) / 10)
        g_ms = window_stats(gw)["median"]
        res["dgemm"][name] = {"M": M, "N": N, "K": K, "ms": g_ms, "TFLOPs": 2.0 * M * N * K / g_ms / 1e9,
                              "frac_of_fp64_matrix_peak": 2.0 * M * N * K / g_ms / 1e9 / 78.6}
    # what a register-resident loop of the same instruction reaches on this chip, and the clocks under that product
    res["mfma_f64_loop_TFLOPs"] = nq.nq_probe_mfma(nq.NQ_F64)
    a = torch.randn((n, m), dtype=torch.float64, device="cuda")
    b = torch.randn((m, r), dtype=torch.float64, device="cuda")
    c = torch.empty((n, r), dtype=torch.float64, device="cuda")
    clocks = ClockSampler()
    t0 = time.perf_counter()
    while clocks.proc is not None and clocks.proc.poll() is None and time.perf_counter() - t0 < 20.0:
        for _ in range(20):
            nq.nq_dgemm(0, 0, n, r, m, 1.0, a, m, b, r, 0.0, c, r)
        torch.cuda.synchronize()
    res["observed_clocks_under_dgemm"] = clocks.read()
    if with_oracle:
        from oracle import lb_admm as O
        t0 = time.perf_counter()
        O.lb_admm(w, u0, v0, 1, 1.0, 20.0, 1e-3, power_iters)
        res["oracle_s_per_iteration"] = time.perf_counter() - t0
        res["oracle_cores"] = os.cpu_count()
    return res


def time_prefill(args, only_layer=None, only_batch=None):
    """Config-5 shapes through nq_binlr_forward at batch 512 / 2048 (TFLOP/s = 2 B r (d_in + d_out) / time)."""
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq
    from paper_2602_06694_amd import synth
    res = {}
    c = synth.CONFIGS[5]
    for li, shp in enumerate(c.block):
        if only_layer and shp.name != only_layer:
            continue
        data = synth.gen_layer(5, 0, li, shp)
        # fp32 outputs (the parity bar's type) and bf16 outputs (what a bf16 model consumes; the fp32 result rounded once more)
        for y_name, y_code, y_torch in (("f32", nq.NQ_F32, torch.float32), ("bf16", nq.NQ_BF16, torch.bfloat16)):
            h = nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out, data.s_in, nq.NQ_BF16, y_code)
            for B in ((only_batch,) if only_batch else c.batches):
                nq.nq_binlr_reserve(h, B)
                xb = synth.gen_layer_x(5, 0, li, shp, B, "bf16", c.outlier_frac)
                x = torch.from_numpy(xb.view(np.int16).copy()).view(torch.bfloat16).cuda()
                y = torch.empty((B, shp.d_out), dtype=y_torch, device="cuda")
                prewarm(lambda: nq.nq_binlr_forward(h, x, y, B), 0.03)
                win = []
                for _ in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    iters = 10
                    e0.record()
                    for _ in range(iters):
                        nq.nq_binlr_forward(h, x, y, B)
                    e1.record()
                    torch.cuda.synchronize()
                    win.append(e0.elapsed_time(e1) / iters)
                ms = window_stats(win)["median"]
                flops = 2.0 * B * shp.r * (shp.d_in + shp.d_out)
                key = f"{shp.name}_{shp.d_out}x{shp.d_in}_B{B}" + ("" if y_name == "f32" else "_y_" + y_name)
                res[key] = {"ms": ms, "ms_windows": window_stats(win), "TFLOP/s": flops / ms / 1e9,
                            "frac_of_f16_mfma_peak": flops / ms / 1e9 / MFMA_F16_PEAK_TFLOPS}
                del x, y
            nq.nq_binlr_destroy(h)
    return res


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2602_06694_amd import binding as nq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    nq.lib()
    if args.case:
        kind = args.case.split(":")
        if kind[0] == "prefill":
            res = time_prefill(args, kind[1], int(kind[2]))
        elif kind[0].startswith("pool_b") and kind[0][6:].isdigit():
            res = time_pool_batch(args.pool, int(kind[0][6:]), two_slice=len(kind) > 1 and kind[1] == "two_slice")
        elif kind[0] in ("stack3", "stack4"):
            res = time_stack(int(kind[0][-1]), 1)
        elif kind[0] in ("chain3", "chain4"):
            res = time_stack_in_dependency_order(int(kind[0][-1]))
        elif kind[0] == "transposed":
            res = time_transposed()
        elif kind[0] == "admm":
            res = time_lb_admm(with_oracle=not args.no_cpu_baseline)
        else:
            print(f"bench.py: unknown --case {args.case}", file=sys.stderr)
            sys.exit(2)
        if args.calibrate_copy:
            a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
            b = torch.empty_like(a)
            b.copy_(a)
            torch.cuda.synchronize()
        print(json.dumps({"case": args.case, "result": res}))
        return
    batch = args.batch
    name, work = build_workload(args)

    handles, xs, ys = [], [], []
    w_bytes = 0
    all_bytes = 0
    y_torch = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.y_dtype]
    y_size = 4 if args.y_dtype == "f32" else 2
    for shp, data, x in work:
        handles.append(nq.nq_binlr_create(shp.d_out, shp.d_in, shp.r, data.U_words, data.V_words, data.s_out,
                                          data.s_in, nq.NQ_BF16, nq.DTYPE_BY_NAME[args.y_dtype]))
        xs.append(torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda())
        ys.append(torch.empty((batch, shp.d_out), dtype=y_torch, device="cuda"))
        wb, ab = algorithmic_bytes(shp, batch, y_size)
        w_bytes += wb
        all_bytes += ab
    plan = nq.nq_plan_create(handles, xs, ys, batch)
    torch.cuda.synchronize()

    prewarm(lambda: nq.nq_plan_forward(plan))
    for _ in range(args.warmup):
        nq.nq_plan_forward(plan)
    torch.cuda.synchronize()
    # EXACTLY `steps` steps are timed for the headline value (window 0); four more windows of the same
    # length follow, and the line also carries their median, minimum and maximum
    clocks = ClockSampler()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        nq.nq_plan_forward(plan)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = e0.elapsed_time(e1) / args.steps
    more_windows = [wall_ms] + timed_windows(lambda: nq.nq_plan_forward(plan), args.steps, 4)
    while clocks.proc is not None and clocks.proc.poll() is None:      # keep the load up until the clocks have been read
        for _ in range(50):
            nq.nq_plan_forward(plan)
        torch.cuda.synchronize()
    observed_clocks = clocks.read()

    # per-kernel durations: a pair of HIP events bound to each launch on its stream (start and stop of the kernel itself,
    # what rocprofv3 reports per dispatch; the dispatch gaps between launches belong to no kernel)
    reps = max(3, min(args.steps, 20))
    per_kernel = np.zeros(4)
    for _ in range(reps):
        per_kernel += np.array(nq.nq_plan_forward_timed(plan))
    per_kernel /= reps
    # the two streaming launches; the slower one is the dominant kernel of the step
    sched = nq.nq_plan_schedules(plan)
    selfq = tuple(w in (32, 33, 34) for w in sched)
    b1 = sum(stage_bytes(shp, batch, y_size, selfq)[0] for shp, _, _ in work)
    b2 = sum(stage_bytes(shp, batch, y_size, selfq)[1] for shp, _, _ in work)
    stages = {"stage1": {"algorithmic_bytes": b1, "ms": per_kernel[1], "GBps": b1 / per_kernel[1] / 1e6},
              "stage2": {"algorithmic_bytes": b2, "ms": per_kernel[3], "GBps": b2 / per_kernel[3] / 1e6}}
    dom = "stage1" if per_kernel[1] >= per_kernel[3] else "stage2"
    achieved = stages[dom]["GBps"]

    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    out = {
        "metric": "effective weight GB/s per layer, decode batch %d" % batch,
        "value": w_bytes / (wall_ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 fixed-point (3 bytes/activation) x 1-bit signs, int32 accumulate; " + {"f32": "fp32", "bf16": "bf16", "f16": "fp16"}[args.y_dtype] + " output",
        "data": "synthetic",
        "config": {"workload": name, "layers_per_step": len(work), "batch": batch,
                   "weight_bytes_per_step": w_bytes, "algorithmic_bytes_per_step": all_bytes},
        "tokens_per_s_per_layer": batch * len(work) / (wall_ms * 1e-3),
        # side figure only: the rate at which a dense bf16 copy of the same layers (2 * d_out * d_in bytes each)
        # would have to stream to finish a step in the same time
        "bf16_dense_equivalent_GBps": sum(2 * shp.d_out * shp.d_in for shp, _, _ in work) / (wall_ms * 1e-3) / 1e9,
        "ms_per_step_hip_events": ev_ms,
        "ms_per_step_windows": window_stats(more_windows),
        "observed_clocks": observed_clocks,
        "kernel_ms": {"quantize_x": per_kernel[0], "stage1": per_kernel[1], "quantize_t": per_kernel[2],
                      "stage2": per_kernel[3]},
        "stages": stages,
        "stage_kernels": [SCHEDULE_KERNEL.get(w, str(w)) for w in sched],
        "roofline": {"bound": "hbm",
                     "kernel": f"{dom} launch ({SCHEDULE_KERNEL.get(sched[0 if dom == 'stage1' else 1], '?')})",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None},
    }
    # what this chip attains on the two roofline resources (context for the fractions of the nominal peaks, not targets)
    if not args.quick:
        hbm = nq.nq_probe_hbm_read(4 << 30, 10, 50)
        out["attainable"] = {"hbm_streaming_read_GBps": hbm,
                             "mfma_f16_dense_TFLOPs": nq.nq_probe_mfma(nq.NQ_F16),
                             "mfma_i8_dense_TOPs": nq.nq_probe_mfma(nq.NQ_I8),
                             "note": "plain read-only kernel over 4 GiB; register-resident matrix-instruction loop"}
        out["roofline"]["frac_of_attainable"] = achieved / hbm
    traffic = measured_traffic(name, dom, out["stage_kernels"][0 if dom == "stage1" else 1])
    if traffic is not None:
        out["roofline"]["traffic"] = traffic
        out["roofline"]["traffic_source"] = ("profiles/stage_kernels_cfg2_pool_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                                             "this workload in a separate run (not measured in this one)")
    nq.nq_plan_destroy(plan)
    for h in handles:
        nq.nq_binlr_destroy(h)
    handles = []
    del xs, ys, plan
    if not args.quick:
        out["extra"] = {"decode_cfg1_single_layer_b1": time_single_layer(1),
                        "decode_cfg2_single_layer_b1": time_single_layer(2),
                        "decode_cfg2_pool_b8": time_pool_batch(args.pool, 8),
                        "decode_cfg2_pool_b8_two_slice_option": time_pool_batch(args.pool, 8, two_slice=True),
                        "decode_llama2_7b_stack_b1": time_stack(3, 1),
                        "decode_llama2_70b_stack_b1": time_stack(4, 1),
                        "decode_llama2_7b_in_dependency_order_b1": time_stack_in_dependency_order(3),
                        "decode_llama2_70b_in_dependency_order_b1": time_stack_in_dependency_order(4),
                        "prefill_config5": time_prefill(args),
                        "lb_admm_cfg2_shape_f64": time_lb_admm(iters=5, with_oracle=not args.no_cpu_baseline)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(work, batch, args.cpu_seconds)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
