#!/usr/bin/env python3
"""Throughput of the whole shuffle path (combine, encode, decode, reduce) on one MI355X.

A step is one pass of the path over one batch of synthetic intermediate values
that are already resident in HBM.  Prints ONE JSON line: logical GB/s of
intermediate values (Q*N*T*elem bytes per step) of the headline workload, the HBM
roofline figure of its dominant kernel measured with events on its stream, the
same figures for the other large workloads and for the accounting in which no
result is shared between the emulated nodes (key "also"), and the CPU oracle
timed on a bounded sample of the headline workload's own inputs as a reported
baseline.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
METRIC = "GB/s of intermediate values through combine+encode+decode; % of HBM peak"

# What the default run measures besides the headline (workload, mode, path).
ALSO = [
    ("cfg5_k24", "f32", "pipeline"),
    ("cfg5_k24", "u32", "pipeline"),
    ("cfg5_k24", "bf16", "pipeline"),
    ("cfg3_gradient", "bf16", "pipeline"),
    ("cfg3_gradient", "f32", "node"),          # per-node-faithful accounting: nothing shared between nodes
    ("cfg3_gradient", "f32", "shuffle+reduce"),
    ("cfg3_gradient", "f32", "map+pipeline"),  # a step that starts from files: Map stand-in, then the one-pass pipeline
]

# HBM bytes per launch of the dominant kernel as the hardware counted them, RECORDED from
# earlier runs of this same command under rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE
# (KiB per dispatch, two runs; the summaries are under profiles/), each scaled by what the
# same counter reads for a device copy of 1 GiB (bench.py --calibrate-copy): FETCH_SIZE reads
# half of the bytes there, so 2.0; WRITE_SIZE reads all of them, so 1.0.  They are not
# measured by the run that prints them.  The figures hold for the kernel sources whose hash
# is recorded with them; for any other source `traffic` is null.
TRAFFIC = {
    ("cfg3_gradient", "f32", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 1420211.0, "write_kib": 1150001.2, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg3_gradient_f32.md"},
    ("cfg5_k24", "f32", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 1043920.8, "write_kib": 462096.0, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg5_k24_f32.md"},
    ("cfg5_k24", "u32", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 1043699.0, "write_kib": 462096.0, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg5_k24_u32.md"},
    ("cfg3_gradient", "bf16", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 707511.3, "write_kib": 575002.7, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg3_gradient_bf16.md"},
    ("cfg5_k24", "bf16", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 531565.0, "write_kib": 249480.0, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg5_k24_bf16.md"},
    ("cfg3_gradient", "f32", "shuffle+reduce"): {
        "source_hash": "0042e45ec8b03434", "fetch_kib": 1050027.0, "write_kib": 3150143.1, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/shuffle_fused_reduce_cfg3_gradient_f32.md"},
    ("jobs_k8", "f32", "shuffle+reduce"): {
        "source_hash": "0042e45ec8b03434", "fetch_kib": 909229.5, "write_kib": 892409.5, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/shuffle_fused_reduce_jobs_k8_f32.md"},
    ("comp_gradient", "f32", "combine+reduce"): {
        "source_hash": "0042e45ec8b03434", "fetch_kib": 1050013.6, "write_kib": 300000.0, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/combine_reduce_comp_gradient_f32.md"},
    ("cfg3_gradient", "f32", "node"): {
        "source_hash": "a1f343c54b1ee29f", "fetch_kib": 2450065.2, "write_kib": 100000.0, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/node_encode_decode_reduce_cfg3_gradient_f32.md"},
    ("cfg3_gradient", "f32", "map+pipeline"): {
        "source_hash": "689605039fbfef14", "fetch_kib": 1450012.0, "write_kib": 2800000.2, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/map_pipeline_fused_cfg3_gradient_f32.md"},
    ("cfg2_k10", "f32", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 11102.3, "write_kib": 7095.8, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg2_k10_f32.md"},
    ("cfg4_k16", "f32", "pipeline"): {
        "source_hash": "4db11b3dcfbb938c", "fetch_kib": 83533.5, "write_kib": 58254.9, "fetch_scale": 2.0, "write_scale": 1.0,
        "profile": "profiles/pipeline_fused_cfg4_k16_f32.md"},
}


# Sources that define the kernels and the launch geometry of each path: a recorded traffic
# figure holds as long as these files are what they were when it was recorded.
PATH_SOURCES = {
    "pipeline": ["pipeline.hip", "common.hpp", "plan.hpp", "plan.cpp"],
    "shuffle+reduce": ["ccdc.hip", "common.hpp", "plan.hpp", "plan.cpp"],
    "combine+reduce": ["ccdc.hip", "common.hpp", "plan.hpp", "plan.cpp"],
    "node": ["node.hip", "common.hpp", "plan.hpp", "plan.cpp"],
    "map+pipeline": ["map.hip", "pipeline.hip", "common.hpp", "plan.hpp", "plan.cpp"],
}


def kernel_source_hash(path):
    import hashlib
    h = hashlib.sha256()
    for f in PATH_SOURCES[path]:
        with open(os.path.join(ROOT, "paper_1805_01993_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, mode, path):
    """(bytes, where they were recorded) or (None, None) when the sources have changed since."""
    t = TRAFFIC.get((workload, mode, path))
    if not t or t["source_hash"] != kernel_source_hash(path):
        return None, None
    return int(1024 * (t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"])), t["profile"]


def elem_bytes(mode):
    return 2 if mode in ("bf16", "f16") else 4


def algorithmic_bytes_shuffle(w, ell, eb=4):
    """Bytes one fused combine+encode+decode launch must move: every needed
    element of V once, every coded packet and every decoded packet once."""
    rounds, r1, W = w.G, w.r + 1, w.W
    reads = rounds * r1 * w.m * W
    writes = rounds * r1 * (ell + W)
    return eb * (reads + writes)


def algorithmic_bytes_pipeline(w, ell, eb=4):
    """Bytes the one-pass pipeline must move: all of V once (every intermediate
    value is either pre-combined for a round or added by its own reducer), every
    coded packet once, the outputs once."""
    return eb * (w.v_elems + w.G * (w.r + 1) * ell + w.Q * w.T)


def host_cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, mode, V_sample, T_sample):
    """The oracle as it stands, single thread, on the first T_sample elements of every
    intermediate value of the inputs the GPU leg ran on (same generator, same seed)."""
    import numpy as np

    import oracle as O

    op = None if w.compression else O.build_plan(w.K, w.r, w.Q, w.N, "paper" if w.jobs else "single")
    V = np.ascontiguousarray(V_sample)
    cp = O.CompressionPlan(w.K, w.r, w.Q, w.N) if w.compression else None
    reps, dt = 0, 0.0
    while dt < 10.0 and reps < 64:         # whole passes over the sample until about 10 s have gone
        t0 = time.perf_counter()
        if w.compression:
            cp.reduce(T_sample, V[0], cp.combine(T_sample, V[0]))
        elif mode == "h32":
            O.run_all_h32(op, T_sample, V)
        elif mode in ("bf16", "f16"):
            O.run_all_h16(op, T_sample, V, mode)
        else:
            O.run_all(op, T_sample, V)
        dt += time.perf_counter() - t0
        reps += 1
    return {"value": round(reps * V.nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"the first {T_sample} of the T={w.T} elements of every intermediate value of the GPU leg's own "
                      f"inputs (generator seed 1; {V.nbytes / 1e6:.0f} MB), same K,r,Q,N, "
                      f"{'combine and reduce' if w.compression else 'all four stages'}, "
                      f"{reps} passes in {dt:.1f} s",
            "host_cpus": os.cpu_count(), "cpu_model": host_cpu_model()}


def measure(torch, L, w, mode, path, steps, warmup, sample_T=0):
    """Time `steps` passes of one workload through one path.  Returns the figures and,
    when sample_T > 0, the host copy of the first sample_T elements of every value."""
    from workloads import generate_torch

    plan = L.Plan(w.K, w.r, w.Q, w.N, jobs=w.jobs, compression=w.compression).bind(w.T, mode).upload()
    sh = plan.shapes()
    eb = elem_bytes(mode)
    dt = {"u32": torch.int32, "bf16": torch.bfloat16, "f16": torch.float16}.get(mode, torch.float32)
    V = generate_torch(w.J, w.N, w.Q, w.T, 1, "f32" if mode == "h32" else mode, sigma=w.sigma, device="cuda")
    X = torch.empty(sh["X"], dtype=dt, device="cuda")
    D = torch.empty(sh["D"], dtype=dt, device="cuda") if path not in ("pipeline", "node", "map+pipeline") else None
    files = theta = None
    if path == "map+pipeline":            # V is made from files by ccdc_map in every step
        files = V
        theta = generate_torch(w.J, 1, w.Q, w.T, 2, "f32" if mode == "h32" else mode, sigma=w.sigma,
                               device="cuda")[:, 0].contiguous()
        V = torch.empty_like(files)
    Phi = torch.empty(sh["Phi"], dtype=dt, device="cuda")
    stream = torch.cuda.current_stream()

    def step(events=None):
        if events is not None:
            events[0].record(stream)
        if path == "pipeline":
            plan.pipeline_fused(V, X, Phi, stream=stream)
            if events is not None:
                events[1].record(stream)
        elif path == "map+pipeline":
            plan.map(files, theta, V, stream=stream)
            if events is not None:
                events[1].record(stream)
            plan.pipeline_fused(V, X, Phi, stream=stream)
        elif path == "node":
            plan.node_encode(-1, V, X, stream=stream)
            if events is not None:
                events[1].record(stream)
            plan.node_decode_reduce(-1, V, X, Phi, stream=stream)
        elif path == "combine+reduce":
            plan.combine(V, D, stream=stream)          # D: the uncoded packets, sent as they are
            if events is not None:
                events[1].record(stream)
            plan.reduce(V, D, Phi, stream=stream)
        else:
            plan.shuffle_fused(V, X, D, stream=stream)
            if events is not None:
                events[1].record(stream)
            plan.reduce(V, D, Phi, stream=stream)
        if events is not None:
            events[2].record(stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = 1e3 * elapsed / steps
    first_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / steps
    second_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / steps
    v_bytes = eb * w.v_elems

    if path == "pipeline":
        alg = algorithmic_bytes_pipeline(w, plan.seg_len, eb)
        kernel, kernel_ms = "k_pipeline (+ k_reduce_final when the rounds are chunked)", {"pipeline_fused": round(first_ms, 4)}
        label = "ccdc_pipeline_fused"
    elif path == "map+pipeline":
        # the map reads every file once and the model once, and writes every intermediate value once
        alg = eb * (2 * w.v_elems + w.J * w.Q * w.T)
        kernel, kernel_ms = "k_map", {"map": round(first_ms, 4), "pipeline_fused": round(second_ms, 4)}
        label = "ccdc_map + ccdc_pipeline_fused (a step that starts from files)"
    elif path == "combine+reduce":
        # every packet reads the files of its batch once and is written once
        ct = plan.compression_tables()
        rows_files = sum(int(n) for n in (ct["batch_first"][1:] - ct["batch_first"][:-1])[ct["pkt_batch"]])
        alg = 4 * w.W * (rows_files + plan.query(L.binding.Q_NROWS))
        kernel, kernel_ms = "k_combine", {"combine": round(first_ms, 4), "reduce": round(second_ms, 4)}
        label = "ccdc_combine + ccdc_reduce (compression-only comparison scheme)"
    elif path == "node":
        # what every node reads for itself: per (round, receiver) the r coded segments meant for it (one packet
        # length) and the r-1 other packets it cancels, pre-combined from m files each; its own files; its outputs
        rows = w.G * (w.r + 1)
        alg = eb * (rows * (w.W + (w.r - 1) * w.m * w.W) + w.r * w.v_elems // w.K + w.J * w.Q * w.T)
        kernel, kernel_ms = "k_node_decode_reduce", {"node_encode": round(first_ms, 4),
                                                     "node_decode_reduce": round(second_ms, 4)}
        label = "ccdc_node_encode + ccdc_node_decode_reduce, every node (per-node-faithful accounting)"
        first_ms = second_ms                           # the dominant kernel is the second call
    else:
        alg = algorithmic_bytes_shuffle(w, plan.seg_len, eb)
        kernel, kernel_ms = "k_shuffle_fused", {"shuffle_fused": round(first_ms, 4), "reduce": round(second_ms, 4)}
        label = "ccdc_shuffle_fused + ccdc_reduce"
    achieved = alg / (first_ms * 1e-3) / 1e9
    traffic, where = measured_traffic(w.name, mode, path)
    sample = None
    if sample_T > 0:
        sample = V[..., :sample_T].contiguous().cpu()
        sample = sample.view(torch.int16).numpy().view("uint16") if eb == 2 else sample.numpy()
        if mode == "u32":
            sample = sample.view("uint32")
    plan.close()
    del V, X, D, Phi, files, theta
    torch.cuda.empty_cache()
    schedule = (f"{w.J} jobs, two-stage schedule" if w.jobs else
                "single job, compression-only comparison scheme" if w.compression else "single job")
    return {
        "workload": f"{w.name}: K={w.K} r={w.r} Q={w.Q} N={w.N} T={w.T} {mode}, {schedule}, "
                    f"{v_bytes / 1e9:.3f} GB of intermediate values per step",
        "path": label, "ms_per_step": ms_per_step, "value": v_bytes / (ms_per_step * 1e-3) / 1e9,
        "kernel": kernel, "kernel_ms": kernel_ms, "dominant_ms": first_ms, "alg": alg, "achieved": achieved,
        "traffic": traffic, "traffic_recorded_in": where, "sample": sample,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3_gradient")
    ap.add_argument("--mode", default=None, help="f32, u32, h32, bf16 or f16 (default: the workload's first mode)")
    ap.add_argument("--path", default="pipeline", choices=["pipeline", "shuffle+reduce", "node", "map+pipeline"],
                    help="pipeline: ccdc_pipeline_fused; shuffle+reduce: ccdc_shuffle_fused then ccdc_reduce; "
                         "node: ccdc_node_encode then ccdc_node_decode_reduce for every node (nothing shared "
                         "between the emulated nodes); map+pipeline: ccdc_map (the Map stand-in, from files) "
                         "then ccdc_pipeline_fused")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true",
                    help="time only the workload named (the default run also times the other large workloads "
                         "and accountings and reports them under the key \"also\")")
    ap.add_argument("--cpu-sample-T", type=int, default=0)
    ap.add_argument("--stream-ceilings", action="store_true",
                    help="run only plain streaming kernels of the array library (fill, copy, add, addcmul on 0.5 GiB "
                         "operands) and print what each sustains: context for the roofline fractions")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of known size (1 GiB read + 1 GiB written per launch): "
                         "what FETCH_SIZE / WRITE_SIZE read for it scales the counters of the other kernels")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU only (all K nodes are emulated on it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1805_01993_amd as L
    from workloads import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    L.load_library()

    if args.stream_ceilings:
        n = 1 << 27                                   # 2^27 fp32 = 0.5 GiB per operand
        a, b, c, d = (torch.full((n,), float(i + 1), dtype=torch.float32, device="cuda") for i in range(4))
        ops = [("fill: 0 reads, 1 write", 1, lambda: d.fill_(1.0)),
               ("copy: 1 read, 1 write", 2, lambda: d.copy_(a)),
               ("add: 2 reads, 1 write", 3, lambda: torch.add(a, b, out=d)),
               ("addcmul: 3 reads, 1 write", 4, lambda: torch.addcmul(a, b, c, out=d)),
               ("sum: 1 read, 0 writes", 1, lambda: a.sum())]
        res = {}
        for name, streams, fn in ops:
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            res[name] = {"ms": round(ms, 4), "GB/s": round(streams * 4 * n / ms / 1e6, 1),
                         "frac_of_peak": round(streams * 4 * n / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        print(json.dumps({"stream_ceilings": res, "operand_bytes": 4 * n, "steps": args.steps}), flush=True)
        return

    if args.calibrate_copy:
        n = 1 << 28                                   # 2^28 fp32 = 1 GiB
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch copy_", "bytes_read_per_launch": 4 * n,
                          "bytes_written_per_launch": 4 * n, "launches": args.warmup + args.steps}), flush=True)
        return

    w = CONFIGS[args.workload]
    mode = args.mode or w.modes[0]
    if w.jobs and args.path in ("pipeline", "map+pipeline"):
        args.path = "shuffle+reduce"      # the one-pass kernel covers single-job plans only
    if w.compression:
        args.path = "combine+reduce"      # the comparison scheme codes nothing
    eb = elem_bytes(mode)
    T_sample = 0
    if not args.no_cpu_baseline:
        T_sample = args.cpu_sample_T or max(4, min(w.T, (1_000_000_000 // (4 * w.J * w.Q * w.N)) // 8 * 8))
    head = measure(torch, L, w, mode, args.path, args.steps, args.warmup, sample_T=T_sample)

    out = {
        "metric": METRIC,
        "value": round(head["value"], 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": mode,
        "data": "synthetic",
        "config": {"workload": head["workload"], "path": head["path"]},
        "pct_hbm_peak_logical": round(100 * head["value"] / HBM_PEAK_GBPS, 2),
        "kernel_ms": head["kernel_ms"],
        "roofline": {"bound": "hbm", "kernel": head["kernel"], "achieved": round(head["achieved"], 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(head["achieved"] / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": head["alg"],
                     "accounting": "per-node-faithful: nothing shared between the emulated nodes" if args.path == "node"
                                   else "shared: every needed element of V read once per launch",
                     "traffic": head["traffic"], "traffic_recorded_in": head["traffic_recorded_in"]},
    }
    if not args.no_also:
        also = {}
        for name, m2, p2 in ALSO:
            if (name, m2, p2) == (w.name, mode, args.path):
                continue
            r = measure(torch, L, CONFIGS[name], m2, p2, args.steps, args.warmup)
            also[f"{name}:{m2}:{p2}"] = {
                "workload": r["workload"], "path": r["path"], "ms_per_step": round(r["ms_per_step"], 4),
                "value": round(r["value"], 2), "kernel": r["kernel"], "ms": round(r["dominant_ms"], 4),
                "kernel_ms": r["kernel_ms"], "algorithmic_bytes": r["alg"], "achieved": round(r["achieved"], 1),
                "frac": round(r["achieved"] / HBM_PEAK_GBPS, 4), "traffic": r["traffic"],
                "traffic_recorded_in": r["traffic_recorded_in"]}
        out["also"] = also
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, mode, head["sample"], T_sample)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
