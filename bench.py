#!/usr/bin/env python3
"""Benchmark of the binary-coding GEMV (inference path of GPTQT) on one MI355X.

Workload (benchmark configs[1]): the OPT-30B-shaped 3-bit layer set at
batch 1 -- 7168x7168 (attention projection), 28672x7168 (fc1), 7168x28672 (fc2),
q = 3, group 128, no offset, synthetic seeded inputs (bcq_synth).  One "step" is
one pass over the three layers, one bcq_gemv each, on one stream.  Weights are
resident in HBM before timing; every step reads a different copy of the packed
weights (the copies total > 1 GiB) so that neither L2 nor the 256 MB memory-side
cache serves them.

Prints ONE JSON line (see README for the fields).  `value` is the
effective weight bandwidth of the whole step; `roofline` is for the dominant
kernel (the 7168x28672 GEMV) from its own timed region; `cpu_baseline` is the
fp64 oracle on the host cores for the same layer set.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak
LAYERS = [("attn_proj", 7168, 7168), ("fc1", 28672, 7168), ("fc2", 7168, 28672)]
DOMINANT = "fc2"
Q, GROUP = 3, 128
PAPER_CONTEXT = ("paper Table IV: GPTQT 3-bit is 1.24x faster than GPTQ 3-bit (and 3.4x faster than fp16) on "
                 "opt-30b, batch 1, NVIDIA RTX A5000, 128-token generation; no per-GEMV time or GB/s is published")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy 10 times (reference kernel of known size for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import bcq_synth
    import paper_2407_02891_amd as bcq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    bcq.lib()  # fails loudly if libbcq.so is missing
    dev = "cuda"

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- build and pack the layer set (not timed) ------------------------------
    layers = {}
    total_bytes = 0
    for name, M, N in LAYERS:
        L = bcq_synth.make_layer(M, N, Q, group=GROUP, offset=False, batch=1, seed=0)
        pl = bcq.PackedLayer(M, N, Q, GROUP, False)
        codes = to_dev(L.codes())
        alpha = to_dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16)
        pl.pack_from(codes, alpha, None)
        torch.cuda.synchronize()
        del codes
        x = to_dev(L.x.view(np.uint16).astype(np.int16)).view(torch.float16)[0]
        y = torch.empty(M, dtype=torch.float16, device=dev)
        layers[name] = dict(L=L, pl=pl, x=x, y=y, bytes=L.weight_bytes(), copies=[pl.packed])
        total_bytes += L.weight_bytes()
    n_copies = max(2, math.ceil(1.25 * 2 ** 30 / total_bytes))
    for name in layers:
        ent = layers[name]
        ent["copies"] += [ent["pl"].packed.clone() for _ in range(n_copies - 1)]
    torch.cuda.synchronize()

    def launch(name, i):
        ent = layers[name]
        pl = ent["pl"]
        bcq.gemv(pl.desc, ent["copies"][i % n_copies], ent["x"], ent["y"],
                 pl.workspace if pl.workspace_bytes else None)

    def step(i):
        for name, _, _ in LAYERS:
            launch(name, i)

    stream = torch.cuda.Stream()  # default priority; all launches and events use it

    def timed(fn, n, first):
        """Time n calls fn(first), fn(first+1), ... with HIP events on `stream`.
        The calls are captured once into a HIP graph (kernel nodes only) and the
        graph is replayed, so the host's launch cost is not what is measured."""
        with torch.cuda.stream(stream):
            if args.no_graph:
                runner = lambda: [fn(first + i) for i in range(n)]
            else:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(n):
                        fn(first + i)
                runner = g.replay
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            torch.cuda.synchronize()
            e0.record(stream)
            runner()
            e1.record(stream)
            stream.synchronize()
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3  # seconds

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            step(i)
        stream.synchronize()

    if args.calibrate_copy:
        src = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: exactly K steps --------------------------------------
    t_steps = timed(step, args.steps, args.warmup)
    ms_per_step = t_steps / args.steps * 1e3
    value_gbs = total_bytes / (t_steps / args.steps) / 1e9

    # ---- per-layer regions (the dominant kernel's gives the roofline) ----------------
    per_layer = {}
    for name, M, N in LAYERS:
        t = timed(lambda i, name=name: launch(name, i), args.steps, args.warmup + 1)
        us = t / args.steps * 1e6
        per_layer[name] = dict(M=M, N=N, us_per_gemv=round(us, 3), weight_bytes=layers[name]["bytes"],
                               weight_GBps=round(layers[name]["bytes"] / us / 1e3, 1),
                               pct_of_hbm_peak=round(layers[name]["bytes"] / us / 1e3 / HBM_PEAK_GBS * 100, 2))
    dom = per_layer[DOMINANT]
    achieved = dom["weight_bytes"] / (dom["us_per_gemv"] * 1e-6) / 1e9
    roofline = dict(bound="hbm", kernel="bcq_gemv_kernel<3,0,4> on 7168x28672", achieved=round(achieved, 1),
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                    bytes_per_launch=dom["weight_bytes"], us_per_launch=dom["us_per_gemv"], traffic=None)
    # HBM bytes per launch measured separately with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE); see profiles/
    traffic_file = os.path.join(ROOT, "profiles", "bcq_gemv_opt30b_q3_hbm_traffic.md")
    if os.path.exists(traffic_file):
        for line in open(traffic_file):
            if line.startswith("hbm_bytes_per_launch_fc2"):
                roofline["traffic"] = float(line.split("=")[1])

    # ---- oracle on the host cores, same layer set --------------------------------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import ref
        t0 = time.perf_counter()
        worst = 0.0
        for name, M, N in LAYERS:
            L = layers[name]["L"]
            y_ref = ref.gemm(L.planes, L.alpha, None, L.x)[0]
            y_gpu = layers[name]["y"].cpu().numpy().astype(np.float64)
            rms = math.sqrt(float(np.mean(y_ref ** 2)))
            err = np.abs(y_gpu - y_ref) / np.maximum(np.abs(y_ref), rms / 64.0)
            worst = max(worst, float(err.max()))
        t_cpu = time.perf_counter() - t0
        cpu = dict(value=round(total_bytes / t_cpu / 1e9, 4), unit="GB/s", cores=ref.num_threads(), kind="oracle",
                   sample="full layer set, one pass (all rows of the 3 layers), fp64 dequant + matvec",
                   seconds=round(t_cpu, 2))
        parity = dict(max_gated_rel_err=worst, tolerance=2e-3)

    out = {
        "metric": "effective weight GB/s (and us per GEMV), 3-bit batch-1 binary-coding GEMV",
        "value": round(value_gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 activations, 1-bit planes x3, f32 accumulate", "data": "synthetic",
        "config": {"workload": "OPT-30B-shaped layer set (7168x7168, 28672x7168, 7168x28672), q=3, group=128, "
                               "batch=1, cold weights (%d rotating copies)" % n_copies,
                   "weight_bytes_per_step": total_bytes, "launch": "graph" if not args.no_graph else "eager"},
        "pct_of_hbm_peak": round(value_gbs / HBM_PEAK_GBS * 100, 2),
        "layers": per_layer, "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
        "context": PAPER_CONTEXT,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
