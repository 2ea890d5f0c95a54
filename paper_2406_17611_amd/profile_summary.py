"""Turns the CSV output of three rocprofv3 runs of bench.py into the short text summaries under profiles/ and
the entry of profiles/hbm_traffic.json that bench.py reports as `roofline.traffic`.

The three runs (on the GPU machine, from /tmp with TMPDIR=/tmp; <out> is any directory; one counter per run):

  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o trace -- python3 bench.py --workload W --steps 3 --warmup 1 --streams 1 --no-cpu-baseline > <out>/trace_bench.json
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- python3 bench.py --workload W --steps 1 --warmup 1 --no-cpu-baseline
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o write -- python3 bench.py --workload W --steps 1 --warmup 1 --no-cpu-baseline

then, anywhere:  python -m paper_2406_17611_amd.profile_summary W <out>

Counter scaling: bench.py issues one plain copy of 256 MiB with the library's copy kernel before its warm-up;
FETCH_SIZE / WRITE_SIZE of every kernel are divided by what the same counter reads per byte of that copy.
The JSON records the hash of the kernel sources the counters were collected on; bench.py warns when the tree's
sources differ.
"""
from __future__ import annotations

import collections
import csv
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CAL_BYTES = 256 * 2**20


def kernel_sources_hash() -> str:
    """SHA-256 over the library's sources (csrc/ and the public header), in name order."""
    h = hashlib.sha256()
    files = sorted(os.listdir(os.path.join(HERE, "csrc")))
    paths = [os.path.join(HERE, "csrc", f) for f in files] + [os.path.join(ROOT, "include", "varco.h")]
    for path in paths:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def _short(name: str) -> str:
    return name.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def _kernel_class(n: str):
    """bench.py's kernel class of a kernel name (None for kernels outside the memory-bound classes)."""
    if n.startswith("spmm_kernel"):
        return "agg_bwd_local" if n.rstrip(">").endswith(" 0") else "agg_fwd"
    for prefix, c in (("spmm_short_rows_kernel", "agg_bwd_local"), ("halo_products_kernel", "agg_bwd_halo"),
                      ("halo_segsum_kernel", "agg_bwd_halo_sum"), ("compress_kernel", "compress"),
                      ("accumulate_returned_kernel", "decompress")):
        if n.startswith(prefix):
            return c
    return None


def _counter(path: str, counter: str):
    per_kernel = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                per_kernel[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return per_kernel


def _find(out_dir: str, suffix: str) -> str:
    for base, _, files in os.walk(out_dir):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(base, f)
    raise FileNotFoundError(f"no *{suffix} under {out_dir}")


def summarise(workload: str, out_dir: str) -> dict:
    prof_dir = os.path.join(ROOT, "profiles")
    with open(os.path.join(out_dir, "trace_bench.json")) as f:
        bench = json.loads(f.read().strip().splitlines()[-1])
    cfg = bench["config"]
    desc = (f"workload {workload} ({cfg['nodes']} nodes, {cfg['directed_entries']} directed entries, {cfg['partitions']} "
            f"partitions, {cfg['conv']} {'-'.join(map(str, cfg['widths']))}, ratio {cfg['ratio']})")
    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 {what} --output-format csv -d <out> -o {name} -- python3 "
           f"/root/repo/bench.py --workload {workload} --steps {{steps}} --warmup 1{{extra}} --no-cpu-baseline")
    with open(_find(out_dir, "trace_kernel_stats.csv")) as f:
        rows = list(csv.DictReader(f))
    with open(os.path.join(prof_dir, f"{workload}_kernel_stats.txt"), "w") as f:
        f.write(f"rocprofv3 kernel statistics, bench.py on {desc}, MI355X;\n1 warm-up + 3 timed + 1 untimed + 3 event-bracketed "
                f"steps (8 steps of launches), all on one stream, so that no two launches overlap and the averages\nbelow are those of "
                f"kernels that have the device to themselves (the headline configuration deals the partitions to two streams).\n"
                f"command: {cmd.format(what='--kernel-trace --stats', name='trace', steps=3, extra=' --streams 1')}\n"
                f"summary written by: python -m paper_2406_17611_amd.profile_summary {workload} <out>\n\n")
        f.write(f"{'kernel':78s} {'calls':>6s} {'total ms':>10s} {'avg us':>10s} {'%':>6s}\n")
        for r in rows:
            n = _short(r["Name"])
            if "kernel" not in n or "at::" in r["Name"]:
                continue
            f.write(f"{n[:78]:78s} {int(r['Calls']):6d} {float(r['TotalDurationNs']) / 1e6:10.2f} "
                    f"{float(r['AverageNs']) / 1e3:10.1f} {float(r['Percentage']):6.2f}\n")
        f.write("\n(build_prow_kernel, build_edges_kernel, the validate_* kernels and the runtime's copyBuffer run once at "
                "registration / upload, outside the timed steps;\ncalibration_copy_kernel is the 256 MiB reference copy "
                "bench.py issues before the warm-up.)\n")
        f.write("\nbench.py's own measurement in the same run (headline: 3 bare steps; per kernel: HIP events around each "
                "launch on the launch stream, 3 further steps):\n")
        f.write(f"  value {bench['value']:.3f} {bench['unit']}, {bench['ms_per_step']:.2f} ms per step "
                f"({bench.get('profiled_pass_ms_per_step') or 0:.2f} in the event-bracketed pass)\n")
        for k, v in bench["kernels"].items():
            extra = f", {100 * v['streaming_frac']:.1f} % on streaming bytes" if "streaming_frac" in v else ""
            f.write(f"  {k:18s} {v['launches_per_step']:5.0f} launches/step  avg {v['avg_launch_ms'] * 1e3:8.1f} us  "
                    f"{v['ms_per_step']:7.2f} ms/step  {v['achieved']:8.1f} {v['unit']} = {100 * v['frac']:.1f} % of "
                    f"{v['bound']} peak{extra}\n")

    fetch = _counter(_find(out_dir, "fetch_counter_collection.csv"), "FETCH_SIZE")
    write = _counter(_find(out_dir, "write_counter_collection.csv"), "WRITE_SIZE")
    cf = sum(fetch["calibration_copy_kernel"]) / len(fetch["calibration_copy_kernel"])
    cw = sum(write["calibration_copy_kernel"]) / len(write["calibration_copy_kernel"])
    sf, sw = cf * 1024 / CAL_BYTES, cw * 1024 / CAL_BYTES
    per_class = collections.defaultdict(lambda: [0.0, 0.0, 0])
    with open(os.path.join(prof_dir, f"{workload}_hbm_traffic.txt"), "w") as f:
        f.write(f"HBM-side traffic per kernel launch from rocprofv3 hardware counters, bench.py on {desc}, MI355X.\n"
                "commands (one counter per run; 1 warm-up + 1 timed + 1 untimed + 1 event-bracketed step):\n"
                f"  {cmd.format(what='--pmc FETCH_SIZE', name='fetch', steps=1, extra='')}\n"
                f"  {cmd.format(what='--pmc WRITE_SIZE', name='write', steps=1, extra='')}\n"
                f"summary written by: python -m paper_2406_17611_amd.profile_summary {workload} <out>\n"
                f"kernel sources (sha256 of csrc/ and include/varco.h): {kernel_sources_hash()}\n\n")
        f.write(f"calibration: the library's plain copy of {CAL_BYTES} bytes (calibration_copy_kernel) reads FETCH_SIZE = "
                f"{cf:.1f} KiB and\nWRITE_SIZE = {cw:.1f} KiB, i.e. the counters report {sf:.4f} x (fetch) and {sw:.4f} x "
                "(write) the bytes in KiB; every figure below is divided by these factors.\n\n")
        f.write(f"{'kernel':78s} {'launches':>8s} {'FETCH MiB/launch':>18s} {'WRITE MiB/launch':>18s}\n")
        for n in sorted(fetch, key=lambda n: -sum(fetch[n])):
            if "kernel" not in n or "at::" in n or n.startswith("__"):
                continue
            fb = sum(fetch[n]) / len(fetch[n]) * 1024 / sf
            wb = sum(write[n]) / len(write[n]) * 1024 / sw if n in write else 0.0
            f.write(f"{n[:78]:78s} {len(fetch[n]):8d} {fb / 2**20:18.1f} {wb / 2**20:18.1f}\n")
            c = _kernel_class(n)
            if c:
                per_class[c][0] += sum(fetch[n]) * 1024 / sf
                per_class[c][1] += sum(write[n]) * 1024 / sw if n in write else 0.0
                if not n.startswith("spmm_short_rows_kernel"):      # second kernel of the same call
                    per_class[c][2] += len(fetch[n])
        f.write("\n(spmm_kernel<..., 1 or 2>: forward aggregation, entries may refer to compressed rows (2: 32-bit offsets "
                "into that buffer), all layers; spmm_kernel<..., 0>: dense rows only (transposed local block). Launches "
                "of one class are averaged together.)\n")

    path = os.path.join(prof_dir, "hbm_traffic.json")
    try:
        with open(path) as f:
            doc = json.load(f)
    except (OSError, ValueError):
        doc = {}
    doc[workload] = {c: {"fetch_bytes_per_launch": fb / n, "write_bytes_per_launch": wb / n, "launches": n}
                     for c, (fb, wb, n) in per_class.items() if n}
    doc.setdefault("kernel_sources_sha256", {})[workload] = kernel_sources_hash()
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    return doc[workload]


if __name__ == "__main__":
    if len(sys.argv) != 3:
        sys.exit(__doc__)
    print(json.dumps(summarise(sys.argv[1], sys.argv[2]), indent=1))
