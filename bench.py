#!/usr/bin/env python3
"""Benchmark of the VARCO layer hot path on one MI355X.

A "step" is one pass of the whole hot path over the workload: for every layer and every partition in turn,
compress boundary rows, aggregate (local rows + compressed halo rows), transform, activate, then the
backward of the same (weight gradients, dM, transposed aggregation, compressed error hand-back, owner-side
accumulation). Inputs are seeded synthetic graphs shaped like the paper's datasets and are resident in HBM
before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--workload large_sage|large_gcn_bf16|medium|medium_bfs16|tiny] [--ratio NUM/DEN]

Prints one JSON line: whole-job GEdges/s (directed CSR entries x layers per step / step time), the roofline
figures of the dominant kernel measured live with HIP events, and the CPU oracle's rate on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix rate
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix rate
HBM_CLASSES = ("compress", "decompress", "agg_fwd", "agg_bwd_local", "agg_bwd_halo", "agg_bwd_halo_sum", "reduce")
MFMA_CLASSES = ("gemm_fwd", "gemm_wgrad", "gemm_dgrad")
DEFAULT_RATIO = {"tiny": (4, 1), "medium": (8, 1), "medium_bfs16": (1584 - 15 * 50, 99), "large_sage": (8, 1),
                 "large_gcn_bf16": (4, 1), "large_sage_bfs8": (8, 1), "large_sage_banded8": (8, 1), "large_gcn_bf16_p4": (4, 1)}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload, kernel_class):
    """HBM bytes per launch of a kernel class from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the same counter reads for the library's plain copy of known size), or None;
    and whether that summary was collected on the kernel sources of this tree (it carries their hash)."""
    from paper_2406_17611_amd.profile_summary import kernel_sources_hash
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            doc = json.load(f)
        rec = doc[workload][kernel_class]
        current = doc.get("kernel_sources_sha256", {}).get(workload) == kernel_sources_hash()
        if not current:
            log(f"[bench] warning: profiles/hbm_traffic.json was collected on other kernel sources than this tree's "
                f"({workload}); the roofline's traffic figure may be stale")
        return rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"], current
    except (OSError, KeyError, ValueError):
        return None, None


def cpu_baseline(w, ratio, budget_s=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the hidden (middle) layer, forward +
    backward, partition after partition in turn until `budget_s` seconds are spent (all partitions when they fit).
    Returns the dict reported under "cpu_baseline"."""
    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import layer as olayer
    from oracle import mask as omask
    from oracle import partition as opart
    from paper_2406_17611_amd import synth

    g = w.graph
    blas_threads = min(os.cpu_count() or 1, 16)
    layer = 1 if len(w.widths) > 2 else 0
    fi, fo = w.widths[layer], w.widths[layer + 1]
    k = omask.keep_count(fi, *ratio)
    h1 = synth.glorot(fi, fo, synth.SEED_WEIGHT, 2 * layer)
    h0 = synth.glorot(fi, fo, synth.SEED_WEIGHT, 2 * layer + 1) if w.conv == "sage" else None
    rng = np.random.default_rng(1)
    wall = cpu = 0.0
    entries = done = 0
    for q in range(w.n_parts):
        # index structures and inputs of the partition: preparation, not part of the layer step
        p = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts, only=[q])[0]
        x = rng.standard_normal((p.n_local, fi)).astype(np.float32)
        z_all = rng.standard_normal((int(p.halo_zrow.max(initial=-1)) + 1, k)).astype(np.float32)
        if w.dtype == "bf16":   # the oracle of the bf16 configuration: fp64 arithmetic on bf16-valued inputs
            from oracle.rounding import round_bf16
            x, z_all = round_bf16(x), round_bf16(z_all)
        dxo = rng.standard_normal((p.n_local, fo)).astype(np.float32)
        with threadpool_limits(limits=blas_threads):
            t0, c0 = time.perf_counter(), time.process_time()
            cols = omask.kept_columns(p.halo_gid, fi, k, synth.MASK_KEY, 0, layer)
            xo, m = olayer.layer_forward(p, x, z_all, cols, h1, h0, olayer.RELU)
            olayer.layer_backward(p, dxo, xo, x, m, cols, h1, h0, olayer.RELU, True)
            wall += time.perf_counter() - t0
            cpu += time.process_time() - c0
        entries += p.nnz
        done += 1
        del p, x, z_all, dxo, xo, m, cols
        if wall >= budget_s:
            break
    busy = cpu / wall
    return {"value": entries / wall / 1e9, "unit": "GEdges/s", "cores": max(1, int(round(busy))), "kind": "oracle",
            "sample": f"partitions 0..{done - 1} of {w.n_parts} in turn, layer {layer + 1} of {len(w.widths) - 1} "
                      f"({fi}->{fo}, k={k}), forward+backward, {entries} directed entries in {wall:.1f} s; numpy/scipy "
                      f"fp64 oracle: {busy:.1f} host threads busy on average (process CPU time / wall time; the dense "
                      f"products may use up to {blas_threads} BLAS threads, the sparse products run on one)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large_sage")
    ap.add_argument("--ratio", default=None, help="num/den, default: the configuration's ratio")
    ap.add_argument("--streams", type=int, default=None,
                    help="HIP streams the partitions of a layer are dealt to in the timed steps (kernels of different "
                         "partitions overlap; the per-kernel pass that follows always uses one stream). Default: 2, "
                         "or 1 for a workload of two partitions (a step of a few hundred microseconds, where the joins cost more than the overlap gains)")
    ap.add_argument("--matmul-terms", type=int, default=None, choices=[0, 2, 3],
                    help="fp32 storage only: form of the dense products (library default 3; 0 = fp32 matrix instructions; "
                         "2 = lower precision, not a valid headline setting)")
    ap.add_argument("--transform-first", action="store_true",
                    help="bf16 storage only: the last layer applies its weights before the aggregation "
                         "(varco_set_layer_order); for comparing the two orders of eq. (2), not the headline setting")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a HIP graph (no per-launch host work; per-kernel timing is not available)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-only", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the partitions of the paper's setting are held in "
                 "one MI355X's memory and processed in turn); --gpus must be 1")

    from paper_2406_17611_amd import synth
    ratio = DEFAULT_RATIO.get(args.workload, (8, 1))
    if args.ratio:
        num, _, den = args.ratio.partition("/")
        ratio = (int(num), int(den or 1))

    t0 = time.time()
    w = synth.make_workload(args.workload)
    g = w.graph
    if args.streams is None:
        args.streams = 1 if w.n_parts <= 2 else 2
    log(f"[bench] workload {w.name}: n={g.n} nnz={g.nnz} P={w.n_parts} conv={w.conv} widths={w.widths} "
        f"ratio={ratio} (generated in {time.time() - t0:.1f}s)")
    if args.cpu_baseline_only:
        print(json.dumps(cpu_baseline(w, ratio)))
        return

    import numpy as np
    import torch

    from paper_2406_17611_amd import binding as vb
    from paper_2406_17611_amd.runner import PartitionedNetwork

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t0 = time.time()
    host = vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts)
    log(f"[bench] partitions built in {time.time() - t0:.1f}s: halo rows {sum(h.n_halo for h in host)}, "
        f"boundary rows {sum(h.n_boundary for h in host)}")
    t0 = time.time()
    L = len(w.widths) - 1
    net = PartitionedNetwork(host, w.widths, w.conv, synth.MASK_KEY, dtype=w.dtype, n_streams=args.streams,
                             transform_first=(L - 1,) if args.transform_first else ())
    if args.matmul_terms is not None:
        net.ctx.set_matmul_terms(args.matmul_terms)
    net.set_inputs(synth.features(g.n, w.widths[0], synth.SEED_FEAT))
    net.set_weights([synth.glorot(w.widths[l], w.widths[l + 1], synth.SEED_WEIGHT, 2 * l) for l in range(L)],
                    [synth.glorot(w.widths[l], w.widths[l + 1], synth.SEED_WEIGHT, 2 * l + 1) for l in range(L)])
    net.set_upstream(synth.upstream_grad(g.n, w.widths[-1], synth.SEED_GRAD))
    torch.cuda.synchronize()
    log(f"[bench] device buffers ready in {time.time() - t0:.1f}s, "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated by torch")

    # one plain copy of known size (256 MiB), outside the timed region: the reference that hardware byte
    # counters of a profiled run are scaled by
    cal_src = torch.ones(64 * 2**20, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    vb.calibration_copy(cal_dst, cal_src)
    del cal_src, cal_dst

    if args.graph:
        graph = net.capture_step(ratio)
        net.ctx.reset_stats()
        net.step(None, ratio)               # one eager step, so that the exchange counters below describe a step
        per_step = net.ctx.stats()
        for s in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = {}
        profiled_ms_per_step = None
        stats = dict(per_step)
        for key in ("fwd_elems", "bwd_elems", "full_fwd_elems", "full_bwd_elems"):
            stats[key] = [v * args.steps for v in per_step[key]]
    else:
        for s in range(args.warmup):
            net.step(s, ratio)
        torch.cuda.synchronize()
        net.ctx.reset_stats()
        # the headline: exactly K steps, nothing but the step's own launches between the two synchronisations
        t0 = time.perf_counter()
        for s in range(args.steps):
            net.step(args.warmup + s, ratio)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        stats = net.ctx.stats()
        # per-kernel table and roofline: a second pass of the same steps with every launch bracketed by HIP events
        # on its launch stream (outside the headline's timed region: the brackets cost about 1 % of a step),
        # and on one stream: with kernels of two partitions overlapping, a launch's bracket would time both
        net.use_streams(1)
        net.step(args.warmup + args.steps, ratio)
        torch.cuda.synchronize()
        net.ctx.profile_enable(True)
        t1 = time.perf_counter()
        for s in range(args.steps):
            net.step(args.warmup + args.steps + 1 + s, ratio)
        torch.cuda.synchronize()
        profiled_ms_per_step = (time.perf_counter() - t1) * 1e3 / args.steps
        prof = net.ctx.profile_read()
        net.ctx.profile_enable(False)
        net.use_streams(args.streams)
    ms_per_step = dt * 1e3 / args.steps
    edges_per_step = L * net.nnz_total
    assert all(torch.isfinite(t).all().item() for t in net.dh1), "non-finite weight gradient"

    kernels = {}
    for name, p in prof.items():
        if not p["launches"]:
            continue
        avg_ms = p["ms"] / p["launches"]
        entry = {"launches_per_step": p["launches"] / args.steps, "ms_per_step": p["ms"] / args.steps,
                 "avg_launch_ms": avg_ms}
        if name in MFMA_CLASSES:
            ach = p["flops"] / p["ms"] / 1e9
            if w.dtype == "bf16":
                peak = MFMA_BF16_PEAK_TFLOPS
            else:
                # fp32 products from bf16 terms: 6 (3) bf16 matrix instructions per algorithmic product-sum
                terms = 3 if args.matmul_terms is None else args.matmul_terms
                peak = {0: MFMA_FP32_PEAK_TFLOPS, 3: MFMA_BF16_PEAK_TFLOPS / 6, 2: MFMA_BF16_PEAK_TFLOPS / 3}[terms]
            entry.update(bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak)
        else:
            ach = p["bytes"] / p["ms"] / 1e6
            entry.update(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS)
            if p["stream_bytes"] != p["bytes"]:
                # the same launches priced on one source-row fetch per entry (no cache between rows)
                entry.update(streaming_achieved=p["stream_bytes"] / p["ms"] / 1e6,
                             streaming_frac=p["stream_bytes"] / p["ms"] / 1e6 / HBM_PEAK_GBS)
        kernels[name] = entry
    roofline = None                     # graph replays and overlapping streams are not bracketed per launch
    if kernels:
        dominant = max((n for n in kernels if n != "reduce"), key=lambda n: kernels[n]["ms_per_step"])
        d = kernels[dominant]
        traffic, current = measured_traffic(w.name, dominant)
        roofline = {"kernel": dominant, "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"],
                    "unit": d["unit"], "frac": d["frac"], "traffic": traffic, "avg_launch_ms": d["avg_launch_ms"]}
        if traffic is not None:
            roofline["traffic_from"] = "profiles/hbm_traffic.json" + ("" if current else " (collected on other kernel sources)")
            roofline["traffic_gbs"] = traffic / d["avg_launch_ms"] / 1e6
        if "streaming_frac" in d:
            roofline["streaming_achieved"] = d["streaming_achieved"]
            roofline["streaming_frac"] = d["streaming_frac"]

    bpe = stats["bytes_per_elem"]
    out = {
        "metric": "GNN layer fwd+bwd GEdges/s at 1 GPU",
        "value": edges_per_step / (ms_per_step * 1e-3) / 1e9,
        "unit": "GEdges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16 storage and matrix products, f32 accumulation",
        "data": "synthetic",
        "config": {"workload": w.name, "nodes": g.n, "directed_entries": g.nnz, "partitions": w.n_parts,
                   "conv": w.conv, "widths": list(w.widths), "ratio": f"{ratio[0]}/{ratio[1]}",
                   "keep": [net.ctx.keep(l) for l in range(L)], "layers": L, "streams": args.streams,
                   "hip_graph": bool(args.graph), "transform_first_layers": [L - 1] if args.transform_first else [],
                   "timed": f"{args.streams} stream{'s' if args.streams > 1 else ''}, " +
                            ("HIP graph replay" if args.graph else "eager launches") + ", no per-launch events; "
                            "per-kernel figures from a separate pass on one stream with HIP events around every launch",
                   "matmul_terms": (3 if args.matmul_terms is None else args.matmul_terms) if w.dtype == "f32" else None,
                   "edges_counted_per_step": edges_per_step},
        "roofline": roofline,
        "kernels": kernels,
        "profiled_pass_ms_per_step": profiled_ms_per_step,
        "exchanged_bytes_per_step": {
            "forward": sum(stats["fwd_elems"]) * bpe // args.steps,
            "backward": sum(stats["bwd_elems"]) * bpe // args.steps,
            "forward_at_ratio_1": sum(stats["full_fwd_elems"]) * bpe // args.steps,
            "backward_at_ratio_1": sum(stats["full_bwd_elems"]) * bpe // args.steps},
    }
    if not args.no_cpu_baseline:
        del net
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, ratio)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
