#!/usr/bin/env python3
"""Benchmark of LoCo's per-step local path on one MI355X.

A step is one pass of the whole path (arXiv 2407.04480, Alg. 1): compensate-quantize
of this worker's gradient shard (steps 1-2) into slot 0 of a receive buffer, then
dequant-reduce of the W payloads in that buffer (step 3).  All inputs are synthetic,
seeded and resident in HBM before the timed region; the error state evolves in place,
so every timed step is a real step.

Prints ONE JSON line: throughput in algorithmic GB/s over the whole step, the
roofline of the dominant kernel (HIP events on the launch stream), and the CPU
oracle timed on this machine's host cores on a bounded sample of the same workload.
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

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE, KiB per
# dispatch), each scaled by what the same counter reads for loco_stream_copy of 2 GiB
# (factor 2.0 for FETCH_SIZE, 1.0 for WRITE_SIZE on this machine).  The profiles/ file of
# the same kernel and workload holds the counters and the commands.
MEASURED_TRAFFIC = {
    ("llama7b_shard_4bit_b256", "loco_compensate_quantize"): 8.8752e9,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce"): 6.9720e9,
    ("llama7b_shard_8bit_b64", "loco_compensate_quantize"): 9.3179e9,
    ("llama7b_shard_8bit_b64", "loco_dequant_reduce"): 1.05485e10,
    ("mixtral_moe_shard_4bit_b128", "loco_compensate_quantize"): 1.48414e10,
    ("mixtral_moe_shard_4bit_b128", "loco_dequant_reduce"): 6.4299e9,
    ("dense70b_shard_4bit_b256", "loco_compensate_quantize"): 2.31829e10,
    ("dense70b_shard_4bit_b256", "loco_dequant_reduce"): 2.76200e10,
    ("llama7b_shard_4bit_b256", "loco_compensate_quantize_fixed"): 3.7904e9,
    ("llama7b_shard_4bit_b256", "loco_compensate_quantize_fixed_f32state"): 8.8441e9,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce_fixed"): 6.7384e9,
    ("llama7b_shard_4bit_b256", "loco_compensate_quantize_clip"): 8.8752e9,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce_sgd"): 1.03411e10,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce_adam"): 2.38180e10,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce_fixed_adam"): 2.35842e10,
    ("llama7b_shard_4bit_b256", "loco_dequant_reduce_bf16"): 5.2874e9,
    ("llama7b_shard_8bit_b64", "loco_compensate_quantize_bf16_scales"): 9.3179e9,
    ("llama7b_shard_8bit_b64", "loco_dequant_reduce_bf16_scales"): 1.03412e10,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_shard_4bit_b256")
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
    ap.add_argument("--no-copy-ceiling", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from a captured HIP graph (two steps per replay); "
                         "reported as graph_replay beside the eager figures, which stay the headline")
    return ap.parse_args()


FIXED_LOG2_S, FIXED_SE_MULT = 19, 4   # the paper's s = 2^19 and s_e = 4s (Sec. 3.1, 3.2)


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(form, w, grads, recv_codes, cstride, recv_scales, nb_full, sample, bytes_cq, bytes_dr):
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
    g_host = workloads.as_numpy_grad(grads[0][:ns])
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


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; payloads of the other workers are resident buffers "
              "on the same device, so --gpus must be 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2407_04480_amd import (loco_code_bytes, loco_compensate_quantize, loco_compensate_quantize_fixed,
                                      loco_dequant_reduce, loco_dequant_reduce_adam, loco_dequant_reduce_bf16,
                                      loco_dequant_reduce_fixed, loco_dequant_reduce_fixed_bf16,
                                      loco_dequant_reduce_fixed_adam, loco_dequant_reduce_fixed_sgd,
                                      loco_dequant_reduce_sgd, loco_error_state8_init, loco_error_state_init,
                                      loco_num_blocks, workloads)
    from paper_2407_04480_amd.binding import (loco_compensate_quantize_fixed_f32state, loco_stream_copy, loco_stream_read, loco_stream_fill, loco_stream_sum2, loco_device_info, loco_compensate_quantize_clip,
                                              loco_compensate_quantize_fixed_clip,
                                              loco_compensate_quantize_bf16_scales,
                                              loco_dequant_reduce_bf16_scales)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path.", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = workloads.by_name(args.workload)
    n, bits, B, W = w.n, w.bits, w.block_size, w.num_workers
    form = args.form
    if args.state == "f32" and (form != "fixed" or args.clip_abs is not None):
        print("bench.py: --state f32 goes with --form fixed and no clipping", file=sys.stderr)
        return 2
    gsz = 2 if w.grad_dtype == torch.bfloat16 else 4
    if form == "block":
        bytes_cq, bytes_dr = workloads.algorithmic_bytes(w)
        names = ("loco_compensate_quantize", "loco_dequant_reduce")
    else:  # gradient + 8-bit state in and out + codes; W payloads of codes + fp32 out
        state_bytes = 1 if args.state == "int8" else 4
        bytes_cq, bytes_dr = gsz + 2 * state_bytes + bits / 8.0, W * bits / 8.0 + 4
        names = ("loco_compensate_quantize_fixed" + ("" if args.state == "int8" else "_f32state"),
                 "loco_dequant_reduce_fixed")
    opt = args.optimizer
    if opt != "none":   # g~ is not written; theta (and m, v) are read and written in place
        bytes_dr += {"sgd": 8, "adam": 24}[opt] - 4
        names = (names[0], names[1] + "_" + opt)
    if args.out == "bf16":
        if opt != "none":
            print("bench.py: --out bf16 has no meaning with a fused optimizer", file=sys.stderr)
            return 2
        bytes_dr -= 2
        names = (names[0], names[1] + "_bf16")
    bf16_steps = args.scales == "bf16"
    clip = args.clip_abs
    if clip is not None:
        names = (names[0] + "_clip", names[1])
    if bf16_steps:
        if form != "block" or opt != "none" or args.out != "f32" or clip is not None:
            print("bench.py: --scales bf16 goes with --form block, no optimizer and fp32 output", file=sys.stderr)
            return 2
        bytes_cq -= 2.0 / B
        bytes_dr -= W * 2.0 / B
        names = (names[0] + "_bf16_scales", names[1] + "_bf16_scales")
    ETA, BETA1, BETA2, DELTA = 1e-4, 0.1, 0.02, 1e-8   # Sec. 4 calls beta1 = 0.1, beta2 in [0.001, 0.05] typical

    # ---- resident inputs: two own gradients (used alternately), W-1 peers' payloads ----
    grads = [workloads.gradient(w, s, device=dev) for s in range(2)]
    cb, nb = loco_code_bytes(n, bits), loco_num_blocks(n, B)
    cstride = (cb + 15) // 16 * 16
    recv_codes = torch.zeros(W * cstride, dtype=torch.uint8, device=dev)
    recv_scales = torch.zeros(W * nb, dtype=torch.bfloat16 if bf16_steps else torch.float32, device=dev)
    own_codes, own_scales = recv_codes[:cb], recv_scales[:nb]
    out = torch.empty(n, dtype=torch.float32 if args.out == "f32" else torch.bfloat16, device=dev) \
        if opt == "none" else None
    theta = torch.randn(n, dtype=torch.float32, device=dev) if opt != "none" else None
    mom = torch.zeros(n, dtype=torch.float32, device=dev) if opt == "adam" else None
    var = torch.zeros(n, dtype=torch.float32, device=dev) if opt == "adam" else None
    stream = torch.cuda.current_stream()

    if form == "block":
        def state_init(e):
            loco_error_state_init(e, stream)

        def cq(g, e, codes, scales):
            if bf16_steps:
                loco_compensate_quantize_bf16_scales(g, e, bits, B, w.beta, False, codes, scales, stream)
            elif clip is not None:
                loco_compensate_quantize_clip(g, clip, e, bits, B, w.beta, False, codes, scales, stream)
            else:
                loco_compensate_quantize(g, e, bits, B, w.beta, False, codes, scales, stream)

        def dr():
            if bf16_steps:
                loco_dequant_reduce_bf16_scales(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "none" and args.out == "bf16":
                loco_dequant_reduce_bf16(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "none":
                loco_dequant_reduce(recv_codes, cstride, recv_scales, nb, W, n, bits, B, out, stream)
            elif opt == "sgd":
                loco_dequant_reduce_sgd(recv_codes, cstride, recv_scales, nb, W, n, bits, B, ETA, theta, stream)
            else:
                loco_dequant_reduce_adam(recv_codes, cstride, recv_scales, nb, W, n, bits, B, ETA, BETA1, BETA2,
                                         DELTA, mom, var, theta, stream)
        err = torch.empty(n, dtype=torch.float32, device=dev)
    else:
        def state_init(e):
            if args.state == "int8":
                loco_error_state8_init(e, stream)
            else:
                loco_error_state_init(e, stream)

        def cq(g, e, codes, scales):
            if args.state == "f32":
                loco_compensate_quantize_fixed_f32state(g, e, bits, FIXED_LOG2_S, w.beta, False, codes, stream)
            elif clip is not None:
                loco_compensate_quantize_fixed_clip(g, clip, e, bits, FIXED_LOG2_S, FIXED_SE_MULT, w.beta, False,
                                                    codes, stream)
            else:
                loco_compensate_quantize_fixed(g, e, bits, FIXED_LOG2_S, FIXED_SE_MULT, w.beta, False, codes, stream)

        def dr():
            if opt == "none" and args.out == "bf16":
                loco_dequant_reduce_fixed_bf16(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, out, stream)
            elif opt == "none":
                loco_dequant_reduce_fixed(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, out, stream)
            elif opt == "sgd":
                loco_dequant_reduce_fixed_sgd(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, ETA, theta, stream)
            else:
                loco_dequant_reduce_fixed_adam(recv_codes, cstride, W, n, bits, FIXED_LOG2_S, ETA, BETA1, BETA2,
                                               DELTA, mom, var, theta, stream)
        err = torch.empty(n, dtype=torch.int8 if args.state == "int8" else torch.float32, device=dev)
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

    for i in range(args.warmup):
        step(i)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    total_s = t1 - t0
    ms_per_step = total_s / args.steps * 1e3

    graph_replay = None
    if args.graph:   # launch-bound sizes: one graph launch instead of two kernel launches per step
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        eager_stream, stream = stream, side
        with torch.cuda.stream(side):
            step(0)
            step(1)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(0)
            step(1)
        stream = eager_stream
        replays = max(1, args.steps // 2)
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        graph_replay = {"steps": 2 * replays, "ms_per_step": (g1 - g0) / (2 * replays) * 1e3,
                        "value": (bytes_cq + bytes_dr) * n / ((g1 - g0) / (2 * replays)) / 1e9, "unit": "GB/s"}
    cq_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    dr_ms = sorted(e[1].elapsed_time(e[2]) for e in events)
    cq_avg, dr_avg = sum(cq_ms) / len(cq_ms), sum(dr_ms) / len(dr_ms)
    step_bytes = (bytes_cq + bytes_dr) * n
    value = step_bytes / (total_s / args.steps) / 1e9

    def kernel_entry(name, per_elem, avg_ms, all_ms):
        gbps = per_elem * n / (avg_ms * 1e-3) / 1e9
        tr = MEASURED_TRAFFIC.get((w.name, name))
        return {"kernel": name, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gbps / HBM_PEAK_GBPS, "traffic": tr, "avg_ms": avg_ms,
                "median_ms": all_ms[len(all_ms) // 2], "min_ms": all_ms[0],
                "algorithmic_bytes_per_launch": per_elem * n}

    k_cq = kernel_entry(names[0], bytes_cq, cq_avg, cq_ms)
    k_dr = kernel_entry(names[1], bytes_dr, dr_avg, dr_ms)
    dominant = k_cq if cq_avg >= dr_avg else k_dr

    # What the memory system sustains for plain streams of 2 GiB in the same run: the ceiling
    # of a pure read stream, a pure write stream, a one-to-one copy and two reads per write.
    copy_gbps, ceilings = None, None
    if not args.no_copy_ceiling:
        nbytes = 1 << 31
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        sink = torch.zeros(16, dtype=torch.uint8, device=dev)
        src.zero_()

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

        copy_gbps = timed(lambda: loco_stream_copy(dst, src, stream), 2 * nbytes)
        ceilings = {"copy": copy_gbps,
                    "read_only": timed(lambda: loco_stream_read(src, sink, stream), nbytes),
                    "write_only": timed(lambda: loco_stream_fill(dst, stream), nbytes)}
        src2 = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        ceilings["two_reads_one_write"] = timed(lambda: loco_stream_sum2(dst, src, src2, stream), 3 * nbytes)
        del src, src2, dst, sink

    cpu = None
    if args.cpu_sample > 0 and opt == "none" and args.out == "f32" and not bf16_steps and clip is None \
            and args.state == "int8":
        # own payload for the sample: one compensate-quantize step from a zero state
        state_init(err)
        cq(grads[0], err, own_codes, own_scales)
        torch.cuda.synchronize()
        cpu = cpu_baseline(form, w, grads, recv_codes, cstride, recv_scales, nb, args.cpu_sample, bytes_cq, bytes_dr)

    line = {
        "metric": METRIC,
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": n, "grad_dtype": str(w.grad_dtype).replace("torch.", ""),
                   "bits": bits, "beta": w.beta, "num_workers": W, "form": form, "optimizer": opt, "out": args.out, "scales": args.scales, "clip_abs": clip,
                   **({"block_size": B} if form == "block" else
                      {"log2_s": FIXED_LOG2_S, "se_mult": FIXED_SE_MULT if args.state == "int8" else None,
                       "state": args.state}),
                   "step": " + ".join(n_[5:] for n_ in names)},
        "elements_per_s": n / (total_s / args.steps),
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "roofline": {k: dominant[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
        | {"kernel": dominant["kernel"]},
        "kernels": [k_cq, k_dr],
        "graph_replay": graph_replay,
        "copy_ceiling_GBps": copy_gbps,
        "stream_ceilings_GBps": ceilings,
        "device": device_report(loco_device_info()),
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
