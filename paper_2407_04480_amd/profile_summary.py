"""Turns rocprofv3 output of bench.py runs into the short summaries under profiles/.

Two steps, so that the raw CSVs (large) never have to leave the GPU machine:

  condense DIR    DIR holds the output of the three profiler runs of one workload (see COMMANDS
                  below): DIR/stats (bench.py under --kernel-trace --stats, its JSON line in
                  DIR/bench.json, its arguments in DIR/args.txt) and DIR/fetch, DIR/write (the
                  plain-C driver loco_traffic_probe under --pmc, its arguments in
                  DIR/probe_args.txt).  Writes DIR/condensed.json: per kernel the call count
                  and durations of the stats run and the mean FETCH_SIZE / WRITE_SIZE per
                  dispatch of the counter runs.
  write FILES...  Each FILE is a condensed.json.  Writes profiles/<entry point>_<workload>.md
                  for the two kernels of the step and updates profiles/traffic.json, the
                  table bench.py reads its `traffic` figures from.
  sweeps FILE     FILE is the JSON line of `bench.py --sweep`; writes profiles/sweeps.md.

The counters are scaled by what they read for the library's plain copy kernel in the same
run (2 GiB read, 2 GiB written): bytes = KiB reported * 1024 * (2 GiB / copy's reading).
They are collected from loco_traffic_probe, a C99 process that makes the same library calls at
the same shape as bench.py: counter collection serialises every dispatch of the process, and
the Python process adds some 10^5 small dispatches of the input generator to the few hundred
of the library.  Kernel names, and therefore launch shapes, are checked to agree between the
two programs.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
COPY_BYTES = 1 << 31
COPY_KERNEL = "stream_kernel<(loco::StreamMode)0"

COMMANDS = """\
    rocprofv3 --kernel-trace --stats -d $O/stats -o st --output-format csv -- python3 bench.py {args} --configs none --steps 10 --warmup 2 --cpu-sample 0
    rocprofv3 --kernel-trace --pmc FETCH_SIZE -d $O/fetch -o pf --output-format csv -- paper_2407_04480_amd/loco_traffic_probe {probe_args}
    rocprofv3 --kernel-trace --pmc WRITE_SIZE -d $O/write -o pw --output-format csv -- paper_2407_04480_amd/loco_traffic_probe {probe_args}"""


def find_one(directory, pattern):
    hits = glob.glob(os.path.join(directory, "**", pattern), recursive=True)
    if len(hits) != 1:
        raise FileNotFoundError(f"expected one {pattern} under {directory}, found {len(hits)}")
    return hits[0]


def short_name(kernel_name: str) -> str:
    """`void loco::cq_kernel<...>(args)` -> `loco::cq_kernel<...>`."""
    name = kernel_name.replace("void ", "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return name[:i]
    return name


def condense(directory: str) -> str:
    stats = {}
    with open(find_one(os.path.join(directory, "stats"), "*kernel_stats.csv")) as fh:
        for row in csv.DictReader(fh):
            if "loco::" not in row["Name"]:
                continue
            stats[short_name(row["Name"])] = {"calls": int(row["Calls"]), "avg_ns": float(row["AverageNs"]),
                                              "min_ns": float(row["MinNs"]), "max_ns": float(row["MaxNs"])}
    counters = collections.defaultdict(lambda: collections.defaultdict(list))
    for sub in ("fetch", "write"):
        with open(find_one(os.path.join(directory, sub), "*counter_collection.csv")) as fh:
            for row in csv.DictReader(fh):
                if "loco::" in row["Kernel_Name"]:
                    counters[short_name(row["Kernel_Name"])][row["Counter_Name"]].append(float(row["Counter_Value"]))
    means = {k: {c: sum(v) / len(v) for c, v in per.items()} for k, per in counters.items()}
    with open(os.path.join(directory, "bench.json")) as fh:
        bench = json.loads([line for line in fh if line.startswith("{")][-1])
    with open(os.path.join(directory, "args.txt")) as fh:
        args = fh.read().strip()
    with open(os.path.join(directory, "probe_args.txt")) as fh:
        probe_args = fh.read().strip()
    out = os.path.join(directory, "condensed.json")
    with open(out, "w") as fh:
        json.dump({"bench_args": args, "probe_args": probe_args, "stats": stats, "counters_KiB_per_dispatch": means, "bench": bench}, fh, indent=1)
    return out


def trace_prefix(entry_point: str) -> tuple:
    """Kernel templates an entry point may launch, as they appear in the trace."""
    if "compensate_quantize" in entry_point:
        if "fixed_f32state" in entry_point:
            return ("loco::fixed_f32_cq_kernel<",)
        return ("loco::fixed_cq_kernel<",) if "fixed" in entry_point else ("loco::cq_kernel<",)
    return ("loco::fixed_dr_kernel<",) if "fixed" in entry_point else ("loco::dr_kernel<", "loco::dr_wide_kernel<")


def write_profiles(files) -> None:
    os.makedirs(PROFILES, exist_ok=True)
    traffic_path = os.path.join(PROFILES, "traffic.json")
    try:
        with open(traffic_path) as fh:
            traffic = json.load(fh)
    except (OSError, ValueError):
        traffic = {}
    loaded = []
    for path in files:
        with open(path) as fh:
            loaded.append((path, json.load(fh)))
    # a kernel that several runs share (the plain compressor under a fused reduce, say) is written
    # by each of them: the run with the plainest command line goes last and is the one that stays
    loaded.sort(key=lambda item: -len(item[1]["bench_args"]))
    for path, data in loaded:
        bench, stats, counters = data["bench"], data["stats"], data["counters_KiB_per_dispatch"]
        workload, n = bench["config"]["workload"], bench["config"]["n"]
        copy = [k for k in counters if COPY_KERNEL in k]
        if not copy:
            raise ValueError(f"{path}: the copy kernel is not in the counter runs")
        fscale = COPY_BYTES / 1024 / counters[copy[0]]["FETCH_SIZE"]
        wscale = COPY_BYTES / 1024 / counters[copy[0]]["WRITE_SIZE"]
        for live in bench["kernels"]:
            entry = live["kernel"]
            names = [k for k in stats if k.startswith(trace_prefix(entry)) and k in counters]
            if len(names) != 1:
                raise ValueError(f"{path}: {entry} maps to {len(names)} kernels of the trace: {names}")
            k = names[0]
            fetch_b = counters[k]["FETCH_SIZE"] * fscale * 1024
            write_b = counters[k]["WRITE_SIZE"] * wscale * 1024
            rd, wr = live["algorithmic_read_bytes_per_launch"], live["algorithmic_write_bytes_per_launch"]
            md = f"{entry}_{workload}.md"
            traffic[f"{entry}|{workload}"] = {"bytes": fetch_b + write_b, "fetch_bytes": fetch_b, "write_bytes": write_b,
                                              "algorithmic_bytes": rd + wr, "source": "profiles/" + md}
            st = stats[k]
            with open(os.path.join(PROFILES, md), "w") as fh:
                fh.write(f"""# {entry} on {workload} (MI355X, one GPU)

Kernel: `{k}`, n = {n} elements per launch.

Commands (run from the repository root on the GPU box after `cd /tmp && export TMPDIR=/tmp`; `$O` is an output folder):

{COMMANDS.format(args=data['bench_args'], probe_args=data['probe_args'])}

`loco_traffic_probe` (paper_2407_04480_amd/csrc/loco_traffic_probe.c, built by `__graft_entry__.build()`) is a C99 process that
makes the same library calls at the same shape; its arguments are N BITS BLOCK WORKERS GRAD FORM OPTIMIZER OUT SCALES CLIP STEPS.
The summary below was made from those CSVs with `python3 -m paper_2407_04480_amd.profile_summary`.

## Duration (`--kernel-trace --stats`, kernel_stats.csv)

| calls | average | min | max |
|---|---|---|---|
| {st['calls']} | {st['avg_ns'] / 1e3:.1f} us | {st['min_ns'] / 1e3:.1f} us | {st['max_ns'] / 1e3:.1f} us |

The same run's bench.py line (HIP events on the launch stream) gives an average of {live['avg_ms'] * 1e3:.1f} us for this
kernel, i.e. {live['achieved']:.0f} GB/s of algorithmic traffic = {100 * live['frac']:.1f} % of the 8000 GB/s HBM peak.
(The call count includes the launches that prepare the peers' payloads and the warm-up steps.)

## HBM traffic (`--pmc`, KiB per dispatch, mean over dispatches)

| counter | this kernel | plain copy of 2 GiB (`loco::stream_kernel`, copy mode) | scale factor | bytes per launch |
|---|---|---|---|---|
| FETCH_SIZE | {counters[k]['FETCH_SIZE']:.1f} | {counters[copy[0]]['FETCH_SIZE']:.1f} | {fscale:.4f} | {fetch_b:.4e} |
| WRITE_SIZE | {counters[k]['WRITE_SIZE']:.1f} | {counters[copy[0]]['WRITE_SIZE']:.1f} | {wscale:.4f} | {write_b:.4e} |

The scale factor is 2 GiB divided by what the counter reads for the copy kernel, which reads 2 GiB and writes 2 GiB.

Algorithmic bytes per launch: read {rd / n:.4f} B/element + write {wr / n:.4f} B/element = {rd + wr:.4e} B.
Measured traffic / algorithmic bytes = {(fetch_b + write_b) / (rd + wr):.4f} (read {fetch_b / rd:.4f}, write {write_b / wr:.4f}).
""")
            print(f"{md}: {live['avg_ms'] * 1e3:.1f} us, frac {live['frac']:.3f}, traffic/algorithmic "
                  f"{(fetch_b + write_b) / (rd + wr):.4f}")
    with open(traffic_path, "w") as fh:
        json.dump(dict(sorted(traffic.items())), fh, indent=1)
        fh.write("\n")


DECOMPOSITION = {1: "quad, scalar/own steps", 2: "quad, lane-loaded steps", 3: "wide 4 B", 4: "wide 8 B", 5: "wide 16 B"}


def table(rows, columns) -> str:
    head = "| " + " | ".join(c for c, _ in columns) + " |\n|" + "---|" * len(columns) + "\n"
    return head + "".join("| " + " | ".join(str(f(r)) for _, f in columns) + " |\n" for r in rows)


def write_sweeps(path: str) -> None:
    with open(path) as fh:
        data = json.loads([line for line in fh if line.startswith("{")][-1])
    sw = data["sweep"]
    pct = ("% of 8 TB/s", lambda r: r["pct_peak"])
    out = ["# Rates off the benchmark configurations (MI355X, one GPU)\n",
           "Made by `python3 bench.py --sweep > $O/sweep.json` on the GPU box and "
           "`python3 -m paper_2407_04480_amd.profile_summary sweeps $O/sweep.json` afterwards.  Every row is the "
           "median of 9 launches after 40 ms of warm-up launches, timed with HIP events on the launch stream; rates are "
           "algorithmic bytes over that time.\n",
           "## Compensate-quantize at the 7B-shard size (842 301 952 elements)\n",
           table(sw["compensate_quantize_7b_shard"],
                 [("gradient", lambda r: r["grad"]), ("form", lambda r: r.get("form", "block")),
                  ("bits", lambda r: r["bits"]), ("block", lambda r: r.get("block_size", "-")),
                  ("ms", lambda r: r["ms"]), ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Compensate-quantize, 4-bit: how the codes leave the wavefront\n",
           "`direct`: 2-byte stores from all 64 lanes (the library's choice); `staged`: gathered in LDS, 16-byte stores "
           "from 16 lanes (`loco_compensate_quantize_staged_codes`).\n",
           table(sw["compensate_quantize_code_store_shapes"],
                 [("block", lambda r: r["block_size"]), ("code stores", lambda r: r["code_stores"]),
                  ("ms", lambda r: r["ms"]), ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Compensate-quantize: wavefronts resident per SIMD (bf16 gradient, 7B-shard size)\n",
           "4 is what `loco_compensate_quantize` runs with; 6 and 8 (all that the kernel's registers allow) through "
           "`loco_compensate_quantize_resident`.\n",
           table(sw.get("compensate_quantize_resident_wavefronts", []),
                 [("bits", lambda r: r["bits"]), ("block", lambda r: r["block_size"]),
                  ("wavefronts per SIMD", lambda r: r["waves_per_simd"]),
                  ("ms", lambda r: r["ms"]), ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Dequant-reduce: every work decomposition at the benchmark sizes\n",
           "`choice` marks what `loco_dequant_reduce` picks by itself.\n",
           table(sw["dequant_reduce_decompositions_benchmark_sizes"],
                 [("n", lambda r: r["n"]), ("bits", lambda r: r["bits"]), ("block", lambda r: r["block_size"]),
                  ("W", lambda r: r["num_workers"]), ("decomposition", lambda r: DECOMPOSITION[r["decomposition"]]),
                  ("choice", lambda r: "yes" if r["library_choice"] else ""), ("ms", lambda r: r["ms"]),
                  ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Dequant-reduce with many workers (52 643 840 elements: the shard of a 7B model over 128 ranks)\n",
           table(sw["dequant_reduce_many_workers"],
                 [("bits", lambda r: r["bits"]), ("block", lambda r: r["block_size"]), ("W", lambda r: r["num_workers"]),
                  ("decomposition", lambda r: DECOMPOSITION[r["decomposition"]]),
                  ("choice", lambda r: "yes" if r["library_choice"] else ""), ("ms", lambda r: r["ms"]),
                  ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## The same reduce when the payload strides are powers of two (2^26 elements, 4-bit, B = 256)\n",
           "The W reads a wavefront issues for one position then fall into one memory channel.\n",
           table(sw["dequant_reduce_power_of_two_strides_2p26"],
                 [("W", lambda r: r["num_workers"]), ("decomposition", lambda r: DECOMPOSITION[r["decomposition"]]),
                  ("choice", lambda r: "yes" if r["library_choice"] else ""), ("ms", lambda r: r["ms"]),
                  ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Fixed-scale reduce with many workers (52 643 840 elements, 4-bit)\n",
           table(sw["dequant_reduce_fixed_many_workers"],
                 [("W", lambda r: r["num_workers"]), ("ms", lambda r: r["ms"]), ("GB/s", lambda r: r["GBps"]), pct]),
           "\n## Shard size (bf16 gradient, 4-bit, B = 256, W = 8; payloads padded by 256 bytes)\n",
           table(sw["shard_size_4bit_b256_w8"],
                 [("n", lambda r: r["n"]), ("CQ ms", lambda r: r["compensate_quantize"]["ms"]),
                  ("CQ % of 8 TB/s", lambda r: r["compensate_quantize"]["pct_peak"]),
                  ("DR ms", lambda r: r["dequant_reduce"]["ms"]), ("DR % of 8 TB/s", lambda r: r["dequant_reduce"]["pct_peak"])]),
           "\nA kernel takes about 6.5 us however small the shard; from 2^25 elements (0.35 GB per call) on, a call runs "
           "within a few points of the full rate.\n",
           "\n## The 2^20-element workload, one step (two kernels), microseconds\n",
           table([sw["gauss_1m_step_us"]], [("eager, from Python", lambda r: r["eager_from_python"]),
                                            ("replayed from a captured HIP graph (two steps per replay)", lambda r: r["hip_graph_replay"])]),
           "\n## Host time per call through the Python binding (4096 elements, 5000 calls)\n",
           table([sw["host_us_per_call_through_the_binding"]],
                 [("pointer checks on, us", lambda r: r["pointer_checks_on"]),
                  ("pointer checks off, us", lambda r: r["pointer_checks_off"])]),
           "\n## The headline measurement six times in a row on one box (GB/s per kernel, 20 steps each)\n",
           table(sw["headline_repeated_6_times_GBps"],
                 [(k, (lambda r, k=k: r[k])) for k in sw["headline_repeated_6_times_GBps"][0]]),
           "\n## Plain streams of 2 GiB in the same run (GB/s)\n",
           table([sw["stream_ceilings_GBps"]], [(k, (lambda r, k=k: r[k])) for k in sw["stream_ceilings_GBps"]])]
    with open(os.path.join(PROFILES, "sweeps.md"), "w") as fh:
        fh.write("\n".join(out))
    print("profiles/sweeps.md written")


def main(argv) -> int:
    if len(argv) >= 2 and argv[0] == "condense":
        for d in argv[1:]:
            print(condense(d))
        return 0
    if len(argv) >= 2 and argv[0] == "write":
        write_profiles(argv[1:])
        return 0
    if len(argv) == 2 and argv[0] == "sweeps":
        write_sweeps(argv[1])
        return 0
    sys.stderr.write(__doc__)
    return 2


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
