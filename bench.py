#!/usr/bin/env python3
"""Benchmark of LoCo's per-step local path on one MI355X.

A step is one pass of the whole path (arXiv 2407.04480, Alg. 1): compensate-quantize
of this worker's gradient shard (steps 1-2) into slot 0 of a receive buffer, then
dequant-reduce of the W payloads in that buffer (step 3).  All inputs are synthetic,
seeded and resident in HBM before the timed region; the error state evolves in place,
so every timed step is a real step.

Prints ONE JSON line.  Its headline fields are the throughput of the headline workload
(the 7B shard, 4-bit, B = 256, W = 8) in algorithmic GB/s over the whole step, the
roofline of the dominant kernel (HIP events on the launch stream), and the CPU oracle
timed on this machine's host cores on a bounded sample of the same workload.  By default
the line also carries "configs": the same measurement, kernel by kernel, for each of
the five benchmark workloads and for Algorithm 1 as printed (global scale, 8-bit state)
on the 7B shard.  `--sweep` prints a different line: rates off the benchmark
configurations (gradient types, block sizes, many workers, work decompositions of the
reduce, host time per call, run-to-run spread).
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

METRIC = "compensate+quantize and dequant-reduce GB/s on one MI355X; % of HBM peak"
HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
HEADLINE = "llama7b_shard_4bit_b256"
FIXED_LOG2_S, FIXED_SE_MULT = 19, 4   # the paper's s = 2^19 and s_e = 4s (Sec. 3.1, 3.2)
ETA, BETA1, BETA2, DELTA = 1e-4, 0.1, 0.02, 1e-8   # Sec. 4 calls beta1 = 0.1, beta2 in [0.001, 0.05] typical

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE), scaled by
# what the same counter reads for a plain copy of known size.  The file is written from the
# profiler's CSVs by `python3 -m paper_2407_04480_amd.profile_summary`; a kernel / workload
# pair that has not been profiled has no entry and reports null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as fh:
            return json.load(fh)
    except (OSError, ValueError):
        return {}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--configs", choices=["auto", "all", "none"], default="auto",
                    help="also measure every benchmark workload and the fixed-scale form ('configs' in the "
                         "line); auto = all for the plain headline run, none when a variant flag is given")
    ap.add_argument("--config-steps", type=int, default=10, help="timed steps of each entry of 'configs'")
    ap.add_argument("--cpu-sample", type=int, default=1 << 30,
                    help="elements of the workload the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--form", choices=["block", "fixed"], default="block",
                    help="block: per-block scales, fp32 error state (the headline path); fixed: Algorithm 1 as "
                         "printed, global scale s = 2^19 and 8-bit error state with s_e = 4s")
    ap.add_argument("--state", choices=["int8", "f32"], default="int8",
                    help="fixed form only: keep the compensation error as 8-bit codes (Algorithm 1 as printed) or "
                         "in fp32 (the paper's ablation row without error compression)")
    ap.add_argument("--optimizer", choices=["none", "sgd", "adam"], default="none",
                    help="fuse the optimizer step of Eq. 9 / Eq. 10 into the reduce (theta, m, v fp32 in place)")
    ap.add_argument("--out", choices=["f32", "bf16"], default="f32",
                    help="type the averaged gradient is written in (bf16: rounded to nearest even)")
    ap.add_argument("--scales", choices=["f32", "bf16"], default="f32",
                    help="block form only: keep the block steps in bf16 (rounded before use)")
    ap.add_argument("--clip-abs", type=float, default=None,
                    help="clip the gradient element-wise to [-c, c] before compensation (Sec. 5.2)")
    ap.add_argument("--decomposition", type=int, default=0,
                    help="block form, plain reduce: work decomposition of the reduce (0 = the library's choice)")
    ap.add_argument("--no-copy-ceiling", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from a captured HIP graph (two steps per replay); "
                         "reported as graph_replay beside the eager figures, which stay the headline")
    ap.add_argument("--sweep", action="store_true",
                    help="print the off-benchmark rates (one JSON line with 'sweep') instead of the benchmark line")
    return ap.parse_args()


class Variant:
    """Which entry points a measurement drives."""

    def __init__(self, form="block", state="int8", optimizer="none", out="f32", scales="f32", clip_abs=None,
                 decomposition=0):
        self.form, self.state, self.optimizer, self.out = form, state, optimizer, out
        self.scales, self.clip_abs, self.decomposition = scales, clip_abs, decomposition

    def plain(self):
        return (self.optimizer == "none" and self.out == "f32" and self.scales == "f32" and self.clip_abs is None
                and self.state == "int8" and self.decomposition == 0)

    def check(self):
        if self.state == "f32" and (self.form != "fixed" or self.clip_abs is not None):
            return "--state f32 goes with --form fixed and no clipping"
        if self.out == "bf16" and self.optimizer != "none":
            return "--out bf16 has no meaning with a fused optimizer"
        if self.scales == "bf16" and (self.form != "block" or self.optimizer != "none" or self.out != "f32"
                                      or self.clip_abs is not None):
            return "--scales bf16 goes with --form block, no optimizer and fp32 output"
        if self.decomposition and (self.form != "block" or not (self.optimizer == "none" and self.out == "f32"
                                                                 and self.scales == "f32")):
            return "--decomposition goes with --form block and the plain fp32 reduce"
        return None


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(form, w, grad0, recv_codes, cstride, recv_scales, nb_full, sample, bytes_cq, bytes_dr):
    """Time the oracle (as it stands) on the first `sample` elements of the workload: one
    compensate-quantize step from a zero state, then the reduce over the W resident payloads."""
    import numpy as np

    import oracle
    from paper_2407_04480_amd import workloads

    B, bits, W = w.block_size, w.bits, w.num_workers
    ns = min(w.n, sample) // (2 * B) * (2 * B)
    if ns == 0:
        return None
    cores = max(1, min(16, os.cpu_count() or 1))
    g_host = workloads.as_numpy_grad(grad0[:ns])
    cb, nb = oracle.code_bytes(ns, bits), oracle.num_blocks(ns, B)
    codes = np.empty((W, cb), np.uint8)
    scales = np.empty((W, nb), np.float32)
    for k in range(W):
        codes[k] = recv_codes[k * cstride:k * cstride + cb].cpu().numpy()
        if form == "block":
            scales[k] = recv_scales[k * nb_full:k * nb_full + nb].cpu().numpy()

    def run(threads):
        t0 = time.perf_counter()
        if form == "block":
            oracle.compensate_quantize(g_host, np.zeros(ns, np.float32), bits, B, w.beta, 0, threads=threads)
        else:
            oracle.fixed_compensate_quantize(g_host, np.zeros(ns, np.int8), bits, FIXED_LOG2_S, FIXED_SE_MULT,
                                             w.beta, 0, threads=threads)
        t1 = time.perf_counter()
        if form == "block":
            oracle.dequant_reduce(codes, scales, W, ns, bits, B, cb, nb, threads=threads)
        else:
            oracle.fixed_dequant_reduce(codes, W, ns, bits, FIXED_LOG2_S, code_stride_bytes=cb, threads=threads)
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    cq1, dr1 = run(1)
    best = None
    for _ in range(3):
        r = run(cores)
        if best is None or r[0] + r[1] < best[0] + best[1]:
            best = r
    cqm, drm = best[0], best[1]
    step_bytes = (bytes_cq + bytes_dr) * ns
    return {
        "value": step_bytes / (cqm + drm) / 1e9,
        "unit": "GB/s",
        "cores": cores,
        "cpu_model": cpu_model(),
        "host_cpus": os.cpu_count(),
        "kind": "oracle",
        "sample": f"first {ns} elements of the shard, one step (compensate-quantize from a zero state + "
                  f"dequant-reduce W={W}), best of 3",
        "seconds": {"compensate_quantize": cqm, "dequant_reduce": drm},
        "elements_per_s": ns / (cqm + drm),
        "single_thread": {"value": step_bytes / (cq1 + dr1) / 1e9, "unit": "GB/s",
                          "seconds": {"compensate_quantize": cq1, "dequant_reduce": dr1}},
    }


def device_report(info):
    """The device's own figures and the HBM peak they imply.  HBM3/3E moves data on both edges
    of a strobe that runs at twice the reported (command) clock: four transfers per clock and pin."""
    info = dict(info)
    info["derived_hbm_peak_GBps"] = 4.0 * info["memory_clock_khz"] * 1e3 * info["memory_bus_bits"] / 8 / 1e9
    return info


def measure(w, v: Variant, steps, warmup, traffic, cpu_sample=0, graph=False):
    """One workload through the path `v` names: `warmup` untimed steps, then exactly `steps` timed
    ones bracketed by synchronisations, with HIP events on the launch stream around each kernel."""
    import torch

    from paper_2407_04480_amd import binding as api
    from paper_2407_04480_amd import workloads

    dev = torch.device("cuda:0")
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    form, opt, clip = v.form, v.optimizer, v.clip_abs
    gsz = 2 if w.grad_dtype == torch.bfloat16 else 4
    # algorithmic bytes per element as (read, write) of each kernel
    bf16_steps = v.scales == "bf16"
    step_bytes_per_elem = (2.0 if bf16_steps else 4.0) / B
    if form == "block":
        rw_cq = (gsz + 4.0, 4.0 + bits / 8.0 + step_bytes_per_elem)
        rw_dr = (W * (bits / 8.0 + step_bytes_per_elem), 4.0)
        names = ["loco_compensate_quantize", "loco_dequant_reduce"]
    else:  # gradient + state in and out + codes; W payloads of codes + fp32 out
        state_bytes = 1.0 if v.state == "int8" else 4.0
        rw_cq = (gsz + state_bytes, state_bytes + bits / 8.0)
        rw_dr = (W * bits / 8.0, 4.0)
        names = ["loco_compensate_quantize_fixed" + ("" if v.state == "int8" else "_f32state"),
                 "loco_dequant_reduce_fixed"]
    if opt != "none":   # g~ is not written; theta (and m, v) are read and written in place
        k_arrays = {"sgd": 1, "adam": 3}[opt]
        rw_dr = (rw_dr[0] + 4.0 * k_arrays, 4.0 * k_arrays)
        names[1] += "_" + opt
    if v.out == "bf16":
        rw_dr = (rw_dr[0], 2.0)
        names[1] += "_bf16"
    if clip is not None:
        names[0] += "_clip"
    if bf16_steps:
        names = [names[0] + "_bf16_scales", names[1] + "_bf16_scales"]
    bytes_cq, bytes_dr = sum(rw_cq), sum(rw_dr)

    # ---- resident inputs: two own gradients (used alternately), W-1 peers' payloads ----
    grads = [workloads.gradient(w, s, device=dev) for s in range(2)]
    cb, nb = api.loco_code_bytes(n, bits), api.loco_num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    recv_codes = torch.zeros(W * cstride, dtype=torch.uint8, device=dev)
    recv_scales = torch.zeros(W * nb, dtype=torch.bfloat16 if bf16_steps else torch.float32, device=dev)
    own_codes, own_scales = recv_codes[:cb], recv_scales[:nb]
    out = torch.empty(n, dtype=torch.float32 if v.out == "f32" else torch.bfloat16, device=dev) \
        if opt == "none" else None
    theta = torch.randn(n, dtype=torch.float32, device=dev) if opt != "none" else None
    mom = torch.zeros(n, dtype=torch.float32, device=dev) if opt == "adam" else None
    var = torch.zeros(n, dtype=torch.float32, device=dev) if opt == "adam" else None
    stream = torch.cuda.current_stream()

    if form == "block":
        def state_init(e):
            api.loco_error_state_init(e, stream)

        def cq(g, e, codes, scales):
            if bf16_steps:
                api.loco_compensate_quantize_bf16_scales(g, e, bits, B, w.beta, False, codes, scales, stream)
            elif clip is not None:
                api.loco_compensate_quantize_clip(g, clip, e, bits, B, w.beta, False, codes, scales, stream)
            else:
                api.loco_compensate_quantize(g, e, bits, B, w.beta, False, codes, scales, stream)

        def dr():
            if bf16_steps:
                api.loco_dequant_reduce_bf16_scales(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "none" and v.out == "bf16":
                api.loco_dequant_reduce_bf16(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "none" and v.decomposition:
                api.loco_dequant_reduce_decomposed(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out,
                                                   v.decomposition, stream)
            elif opt == "none":
                api.loco_dequant_reduce(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "sgd":
                api.loco_dequant_reduce_sgd(recv_codes, cstride, recv_scales, nb, W, n, bits, B, ETA, theta, stream)
            else:
                api.loco_dequant_reduce_adam(recv_codes, cstride, recv_scales, nb, W, n, bits, B, ETA, BETA1, BETA2,
                                             DELTA, mom, var, theta, stream)
        err = torch.empty(n, dtype=torch.float32, device=dev)
    else:
        def state_init(e):
            if v.state == "int8":
                api.loco_error_state8_init(e, stream)
            else:
                api.loco_error_state_init(e, stream)

        def cq(g, e, codes, scales):
            if v.state == "f32":
                api.loco_compensate_quantize_fixed_f32state(g, e, bits, FIXED_LOG2_S, w.beta, False, codes, stream)
            elif clip is not None:
                api.loco_compensate_quantize_fixed_clip(g, clip, e, bits, FIXED_LOG2_S, FIXED_SE_MULT, w.beta, False,
                                                        codes, stream)
            else:
                api.loco_compensate_quantize_fixed(g, e, bits, FIXED_LOG2_S, FIXED_SE_MULT, w.beta, False, codes,
                                                   stream)

        def dr():
            if opt == "none" and v.out == "bf16":
                api.loco_dequant_reduce_fixed_bf16(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, out, stream)
            elif opt == "none":
                api.loco_dequant_reduce_fixed(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, out, stream)
            elif opt == "sgd":
                api.loco_dequant_reduce_fixed_sgd(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, ETA, theta, stream)
            else:
                api.loco_dequant_reduce_fixed_adam(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, ETA, BETA1, BETA2,
                                                   DELTA, mom, var, theta, stream)
        err = torch.empty(n, dtype=torch.int8 if v.state == "int8" else torch.float32, device=dev)
    state_init(err)
    tmp_err = torch.empty_like(err)
    for k in range(1, W):
        gk = workloads.gradient(w, 0, worker=k, device=dev)
        state_init(tmp_err)
        cq(gk, tmp_err, recv_codes[k * cstride:k * cstride + cb], recv_scales[k * nb:(k + 1) * nb])
        del gk
    del tmp_err
    torch.cuda.synchronize()

    def step(i, ev=None):
        g = grads[i & 1]
        if ev is not None:
            ev[0].record(stream)
        cq(g, err, own_codes, own_scales)
        if ev is not None:
            ev[1].record(stream)
        dr()
        if ev is not None:
            ev[2].record(stream)

    for i in range(warmup):
        step(i)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_s = t1 - t0

    graph_replay = None
    if graph:   # launch-bound sizes: one graph launch instead of two kernel launches per step
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        eager_stream, stream = stream, side
        with torch.cuda.stream(side):
            step(0)
            step(1)
        torch.cuda.synchronize()
        cuda_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cuda_graph, stream=side):
            step(0)
            step(1)
        stream = eager_stream
        replays = max(1, steps // 2)
        cuda_graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(replays):
            cuda_graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        graph_replay = {"steps": 2 * replays, "ms_per_step": (g1 - g0) / (2 * replays) * 1e3,
                        "value": (bytes_cq + bytes_dr) * n / ((g1 - g0) / (2 * replays)) / 1e9, "unit": "GB/s"}

    cq_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    dr_ms = sorted(e[1].elapsed_time(e[2]) for e in events)

    def kernel_entry(name, rw, all_ms):
        per_elem = sum(rw)
        avg_ms = sum(all_ms) / len(all_ms)
        gbps = per_elem * n / (avg_ms * 1e-3) / 1e9
        tr = traffic.get(f"{name}|{w.name}")
        return {"kernel": name, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gbps / HBM_PEAK_GBPS, "traffic": tr["bytes"] if tr else None,
                "traffic_source": tr["source"] if tr else None, "avg_ms": avg_ms,
                "median_ms": all_ms[len(all_ms) // 2], "min_ms": all_ms[0],
                "algorithmic_bytes_per_launch": per_elem * n,
                "algorithmic_read_bytes_per_launch": rw[0] * n, "algorithmic_write_bytes_per_launch": rw[1] * n}

    k_cq = kernel_entry(names[0], rw_cq, cq_ms)
    k_dr = kernel_entry(names[1], rw_dr, dr_ms)
    step_bytes = (bytes_cq + bytes_dr) * n
    result = {
        "workload": w.name, "form": form, "n": n, "grad_dtype": str(w.grad_dtype).replace("torch.", ""),
        "bits": bits, "num_workers": W, "beta": w.beta,
        **({"block_size": B} if form == "block" else
           {"log2_s": FIXED_LOG2_S, "se_mult": FIXED_SE_MULT if v.state == "int8" else None, "state": v.state}),
        "steps": steps, "warmup": warmup, "ms_per_step": total_s / steps * 1e3,
        "value": step_bytes / (total_s / steps) / 1e9, "unit": "GB/s",
        "elements_per_s": n / (total_s / steps), "kernels": [k_cq, k_dr], "graph_replay": graph_replay,
        "step": " + ".join(x[5:] for x in names),
    }
    if form == "block" and opt == "none" and v.out == "f32" and not bf16_steps:
        result["reduce_decomposition"] = v.decomposition or api.loco_dequant_reduce_decomposition(W, bits, B)

    cpu = None
    if cpu_sample > 0 and v.plain():
        # own payload for the sample: one compensate-quantize step from a zero state
        state_init(err)
        cq(grads[0], err, own_codes, own_scales)
        torch.cuda.synchronize()
        cpu = cpu_baseline(form, w, grads[0], recv_codes, cstride, recv_scales, nb, cpu_sample, bytes_cq, bytes_dr)
    return result, cpu


def stream_ceilings():
    """What the memory system sustains for plain streams of 2 GiB in this run: a pure read, a pure
    write, a one-to-one copy, two reads per write, and the HIP runtime's own device-to-device copy."""
    import torch

    from paper_2407_04480_amd import binding as api

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    nbytes = 1 << 31
    src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
    src2 = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)

    def timed(fn, moved):
        for _ in range(2):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(10):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return moved * 10 / (a.elapsed_time(b) * 1e-3) / 1e9

    return {"copy": timed(lambda: api.loco_stream_copy(dst, src, stream), 2 * nbytes),
            "read_only": timed(lambda: api.loco_stream_read(src, sink, stream), nbytes),
            "write_only": timed(lambda: api.loco_stream_fill(dst, stream), nbytes),
            "two_reads_one_write": timed(lambda: api.loco_stream_sum2(dst, src, src2, stream), 3 * nbytes),
            "three_arrays_updated_in_place": timed(lambda: api.loco_stream_update3(dst, src, src2, stream), 6 * nbytes),
            "runtime_copy_hipMemcpyDtoDAsync": timed(lambda: api.loco_runtime_copy(dst, src, stream), 2 * nbytes)}


def release():
    import gc

    import torch
    gc.collect()
    torch.cuda.empty_cache()


def config_entry(result):
    keep = ("workload", "form", "n", "grad_dtype", "bits", "block_size", "log2_s", "se_mult", "state", "num_workers",
            "steps", "warmup", "ms_per_step", "value", "unit", "elements_per_s", "reduce_decomposition")
    entry = {k: result[k] for k in keep if k in result}
    if sum(k["algorithmic_bytes_per_launch"] for k in result["kernels"]) < 256e6:
        entry["note"] = ("the whole step moves less than the 256 MB memory-side cache and each kernel runs a few "
                         "microseconds: bound by launches, not by HBM; a parity workload, not a bandwidth figure")
    entry["kernels"] = [{k: kern[k] for k in ("kernel", "avg_ms", "min_ms", "achieved", "frac", "traffic",
                                              "traffic_source", "algorithmic_bytes_per_launch")}
                        for kern in result["kernels"]]
    return entry


def sweep(args):
    """Rates off the benchmark configurations, all through the C ABI."""
    import torch

    from paper_2407_04480_amd import binding as api
    from paper_2407_04480_amd import workloads

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()

    def median_ms(fn, reps=9, warm_ms=40.0):
        # keep the GPU busy for a while first: after an idle stretch (host-side set-up) the first
        # launches of a short burst run at reduced clocks and read 10-20 % slow
        t0 = time.perf_counter()
        while True:
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
            if (time.perf_counter() - t0) * 1e3 >= warm_ms:
                break
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        return ms[len(ms) // 2]

    def rate(per_elem, n, ms):
        gbps = per_elem * n / (ms * 1e-3) / 1e9
        return {"ms": round(ms, 4), "GBps": round(gbps, 1), "pct_peak": round(100 * gbps / HBM_PEAK_GBPS, 1)}

    out = {}
    # ---- compensate-quantize: gradient type x bit width x block size at the 7B-shard size ----
    w7 = workloads.by_name(HEADLINE)
    n = w7.n
    g16 = workloads.gradient(w7, 0, device=dev)
    g32 = g16.float()
    err = torch.zeros(n, dtype=torch.float32, device=dev)
    codes = torch.empty(n, dtype=torch.uint8, device=dev)
    scales = torch.empty(n // 32, dtype=torch.float32, device=dev)
    table = []
    for g in (g32, g16):
        for bits, B in ((4, 256), (8, 64), (4, 128), (4, 32), (8, 512)):
            ms = median_ms(lambda: api.loco_compensate_quantize(g, err, bits, B, 0.25, False, codes, scales, stream))
            per = g.element_size() + 8 + bits / 8 + 4 / B
            table.append({"grad": str(g.dtype).replace("torch.", ""), "bits": bits, "block_size": B,
                          **rate(per, n, ms)})
    err8 = torch.zeros(n, dtype=torch.int8, device=dev)
    for g in (g32, g16):
        ms = median_ms(lambda: api.loco_compensate_quantize_fixed(g, err8, 4, FIXED_LOG2_S, FIXED_SE_MULT, 0.25, False,
                                                                 codes, stream))
        table.append({"grad": str(g.dtype).replace("torch.", ""), "bits": 4, "form": "fixed",
                      **rate(g.element_size() + 2 + 0.5, n, ms)})
    out["compensate_quantize_7b_shard"] = table
    # 4-bit codes: direct 2-byte stores from every lane against 16-byte stores staged through LDS
    staged = []
    for g in (g16,):
        for B in (256, 128):
            for name, fn in (("direct", api.loco_compensate_quantize), ("staged", api.loco_compensate_quantize_staged_codes)):
                ms = median_ms(lambda: fn(g, err, 4, B, 0.25, False, codes, scales, stream))
                staged.append({"grad": "bfloat16", "bits": 4, "block_size": B, "code_stores": name,
                               **rate(g.element_size() + 8 + 0.5 + 4 / B, n, ms)})
    out["compensate_quantize_code_store_shapes"] = staged
    # resident wavefronts per SIMD: the library's 4 against 6 and the 8 the registers allow
    resident = []
    for bits, B in ((4, 256), (8, 64), (4, 128), (4, 32)):
        for waves in (4, 6, 8):
            ms = median_ms(lambda: api.loco_compensate_quantize_resident(g16, err, bits, B, 0.25, False, codes, scales,
                                                                         waves, stream))
            resident.append({"grad": "bfloat16", "bits": bits, "block_size": B, "waves_per_simd": waves,
                             **rate(g16.element_size() + 8 + bits / 8 + 4 / B, n, ms)})
    out["compensate_quantize_resident_wavefronts"] = resident
    del g16, g32, err, err8, codes, scales
    release()

    # ---- dequant-reduce: decompositions at the benchmark sizes and with many workers ----
    def reduce_rows(n, bits, B, W, decompositions):
        cb, nb = api.loco_code_bytes(n, bits), api.loco_num_blocks(n, B)
        cs = (cb + 15) // 16 * 16
        gen = torch.Generator(device=dev).manual_seed(1)
        rc = torch.randint(0, 256, (W * cs,), dtype=torch.uint8, device=dev, generator=gen)
        rs = torch.rand(W * nb, dtype=torch.float32, device=dev, generator=gen) * 1e-3 + 1e-6
        o = torch.empty(n, dtype=torch.float32, device=dev)
        per = W * (bits / 8 + 4 / B) + 4
        rows = []
        auto = api.loco_dequant_reduce_decomposition(W, bits, B)
        for d in decompositions:
            try:
                ms = median_ms(lambda: api.loco_dequant_reduce_decomposed(rc, cs, rs, nb, W, n, bits, B, o, d, stream))
            except api.LocoError:
                continue
            rows.append({"n": n, "bits": bits, "block_size": B, "num_workers": W, "decomposition": d,
                         "library_choice": d == auto, **rate(per, n, ms)})
        del rc, rs, o
        release()
        return rows

    rows = []
    for n_, bits, B, W in ((w7.n, 4, 256, 8), (w7.n, 8, 64, 8), (1409286144, 4, 128, 1), (2200000000, 4, 256, 16)):
        rows += reduce_rows(n_, bits, B, W, (1, 2, 3, 4, 5))
    out["dequant_reduce_decompositions_benchmark_sizes"] = rows
    rows = []
    n128 = 52643840          # the 7B model's flat gradient over 128 ranks, rounded down to whole tiles
    for bits in (4, 8):
        for B in (64, 256):
            for W in (16, 32, 64, 128):
                rows += reduce_rows(n128, bits, B, W, (1, 2, 3, 4, 5))
    out["dequant_reduce_many_workers"] = rows
    rows = []                # payload strides that are powers of two: the W reads of a wavefront share a channel
    for W in (16, 32, 128):
        rows += reduce_rows(1 << 26, 4, 256, W, (1, 5))
    out["dequant_reduce_power_of_two_strides_2p26"] = rows
    rows = []
    nn = n128
    for W in (16, 32, 64, 128):
        cs = nn // 2
        rc = torch.randint(0, 256, (W * cs,), dtype=torch.uint8, device=dev)
        o = torch.empty(nn, dtype=torch.float32, device=dev)
        ms = median_ms(lambda: api.loco_dequant_reduce_fixed(rc, cs, W, nn, 4, FIXED_LOG2_S, o, stream))
        rows.append({"n": nn, "bits": 4, "form": "fixed", "num_workers": W, **rate(W * 0.5 + 4, nn, ms)})
        del rc, o
        release()
    out["dequant_reduce_fixed_many_workers"] = rows

    # ---- shard size: where a call stops being bound by the launch ----
    rows = []
    for log2n in range(20, 29):
        nn = 1 << log2n
        w_ = workloads.Workload(f"size_2p{log2n}", "gauss", nn, torch.bfloat16, 4, 256, num_workers=8,
                                segments=(("all", 0, nn),))
        gk = workloads.gradient(w_, 0, device=dev)
        ek = torch.zeros(nn, dtype=torch.float32, device=dev)
        cbk, nbk = api.loco_code_bytes(nn, 4), api.loco_num_blocks(nn, 256)
        csk = cbk + 256                       # payloads padded: strides of 2^k bytes share a memory channel
        rck = torch.zeros(8 * csk, dtype=torch.uint8, device=dev)
        rsk = torch.rand(8 * (nbk + 8), dtype=torch.float32, device=dev) * 1e-3
        ok = torch.empty(nn, dtype=torch.float32, device=dev)
        ms_cq = median_ms(lambda: api.loco_compensate_quantize(gk, ek, 4, 256, 0.25, False, rck[:cbk], rsk[:nbk], stream))
        ms_dr = median_ms(lambda: api.loco_dequant_reduce(rck, csk, rsk, nbk + 8, 8, nn, 4, 256, ok, stream))
        rows.append({"n": nn, "compensate_quantize": rate(10.515625, nn, ms_cq), "dequant_reduce": rate(8.125, nn, ms_dr)})
        del gk, ek, rck, rsk, ok
        release()
    out["shard_size_4bit_b256_w8"] = rows
    small, _cpu = measure(workloads.by_name("gauss_1m"), Variant(), 200, 20, load_traffic(), graph=True)
    out["gauss_1m_step_us"] = {"eager_from_python": round(small["ms_per_step"] * 1e3, 2),
                               "hip_graph_replay": round(small["graph_replay"]["ms_per_step"] * 1e3, 2)}

    # ---- host time per call (a launch-bound size), with and without the pointer checks ----
    ns = 1 << 12
    g = torch.zeros(ns, dtype=torch.bfloat16, device=dev)
    e = torch.zeros(ns, dtype=torch.float32, device=dev)
    c = torch.zeros(ns // 2, dtype=torch.uint8, device=dev)
    s = torch.zeros(ns // 256, dtype=torch.float32, device=dev)
    host = {}
    for checks in (True, False):
        api.loco_set_pointer_checks(checks)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5000):
            api.loco_compensate_quantize(g, e, 4, 256, 0.25, False, c, s, stream)
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        host["pointer_checks_on" if checks else "pointer_checks_off"] = round((t1 - t0) / 5000 * 1e6, 2)
    api.loco_set_pointer_checks(True)
    out["host_us_per_call_through_the_binding"] = host

    # ---- run-to-run spread of the headline measurement on this machine ----
    traffic = load_traffic()
    runs = []
    for _ in range(6):
        r, _cpu = measure(w7, Variant(), 20, 3, traffic)
        runs.append({k["kernel"]: round(k["achieved"], 1) for k in r["kernels"]})
        release()
    out["headline_repeated_6_times_GBps"] = runs
    out["stream_ceilings_GBps"] = {k: round(x, 1) for k, x in stream_ceilings().items()}
    print(json.dumps({"sweep": out, "device": device_report(api.loco_device_info()), "peak_GBps": HBM_PEAK_GBPS}))
    return 0


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; payloads of the other workers are resident buffers "
              "on the same device, so --gpus must be 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2407_04480_amd import binding as api
    from paper_2407_04480_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path.", file=sys.stderr)
        return 2
    torch.cuda.set_device(torch.device("cuda:0"))
    if args.sweep:
        return sweep(args)

    v = Variant(args.form, args.state, args.optimizer, args.out, args.scales, args.clip_abs, args.decomposition)
    problem = v.check()
    if problem:
        print("bench.py: " + problem, file=sys.stderr)
        return 2
    traffic = load_traffic()
    w = workloads.by_name(args.workload)
    main_result, cpu = measure(w, v, args.steps, args.warmup, traffic, cpu_sample=args.cpu_sample, graph=args.graph)
    release()

    want_all = args.configs == "all" or (args.configs == "auto" and args.workload == HEADLINE and v.plain()
                                         and v.form == "block")
    configs = None
    if want_all:
        configs = []
        for name in workloads.WORKLOAD_NAMES:
            if name == w.name and v.plain() and v.form == "block":
                configs.append(config_entry(main_result))     # the headline itself, as timed above
                continue
            r, _ = measure(workloads.by_name(name), Variant(), args.config_steps, 2, traffic)
            configs.append(config_entry(r))
            release()
        r, _ = measure(workloads.by_name(HEADLINE), Variant(form="fixed"), args.config_steps, 2, traffic)
        configs.append(config_entry(r))
        release()

    ceilings = None if args.no_copy_ceiling else stream_ceilings()
    k_cq, k_dr = main_result["kernels"]
    dominant = k_cq if k_cq["avg_ms"] >= k_dr["avg_ms"] else k_dr
    line = {
        "metric": METRIC,
        "value": main_result["value"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_result["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "grad_dtype": main_result["grad_dtype"], "bits": w.bits,
                   "beta": w.beta, "num_workers": w.num_workers, "form": v.form, "optimizer": v.optimizer,
                   "out": v.out, "scales": v.scales, "clip_abs": v.clip_abs,
                   **({"block_size": w.block_size} if v.form == "block" else
                      {"log2_s": FIXED_LOG2_S, "se_mult": FIXED_SE_MULT if v.state == "int8" else None,
                       "state": v.state}),
                   "reduce_decomposition": main_result.get("reduce_decomposition"),
                   "step": main_result["step"]},
        "elements_per_s": main_result["elements_per_s"],
        "pct_hbm_peak": 100.0 * main_result["value"] / HBM_PEAK_GBPS,
        "roofline": {k: dominant[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
        | {"kernel": dominant["kernel"], "traffic_source": dominant["traffic_source"]},
        "kernels": main_result["kernels"],
        "configs": configs,
        "graph_replay": main_result["graph_replay"],
        "copy_ceiling_GBps": ceilings["copy"] if ceilings else None,
        "stream_ceilings_GBps": ceilings,
        "device": device_report(api.loco_device_info()),
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
