#!/usr/bin/env python3
"""Benchmark of the binary-coding GEMV (inference path of GPTQT) on one MI355X.

Default workload: the OPT-30B-shaped 3-bit layer set at
batch 1 -- 7168x7168 (attention projection), 28672x7168 (fc1), 7168x28672 (fc2),
q = 3, group 128, no offset, synthetic seeded inputs (bcq_synth).  One "step" is
one pass over the layers, one bcq_gemv each, on one stream.  Weights are
resident in HBM before timing; every step reads a different copy of the packed
weights (the copies of the largest layer alone total at least 1 GiB) so that
neither L2 nor the 256 MB memory-side cache serves them.

Other workloads (--workload): `llama70b_block` = the seven GEMVs of a
Llama-2-70B-shaped decoder block in sequence; `llama70b_block_fused` = the same
weights with the projections that share their input (q/k/v; gate/up) packed into
one blob each with bcq_pack_rows, four GEMVs per step.  --q selects 2 or 3 planes.

Prints ONE JSON line (the fields are described in README.md).  `value` is the
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
GROUP = 128
# name -> (launches, dominant launch, description); a launch = (name, [(part name, rows), ...], N)
WORKLOADS = {
    "opt30b": ([("attn_proj", [("attn_proj", 7168)], 7168), ("fc1", [("fc1", 28672)], 7168),
                ("fc2", [("fc2", 7168)], 28672)], "fc2",
               "OPT-30B-shaped layer set (7168x7168, 28672x7168, 7168x28672)"),
    "opt66b": ([("attn_proj", [("attn_proj", 9216)], 9216), ("fc1", [("fc1", 36864)], 9216),
                ("fc2", [("fc2", 9216)], 36864)], "fc2",
               "OPT-66B-shaped layer set (9216x9216, 36864x9216, 9216x36864)"),
    "llama70b_block": ([("q", [("q", 8192)], 8192), ("k", [("k", 1024)], 8192), ("v", [("v", 1024)], 8192),
                        ("o", [("o", 8192)], 8192), ("gate", [("gate", 28672)], 8192),
                        ("up", [("up", 28672)], 8192), ("down", [("down", 8192)], 28672)], "down",
                       "Llama-2-70B-shaped decoder block, 7 GEMVs in sequence (q, k, v, o, gate, up, down)"),
    "llama70b_block_fused": ([("qkv", [("q", 8192), ("k", 1024), ("v", 1024)], 8192), ("o", [("o", 8192)], 8192),
                              ("gate_up", [("gate", 28672), ("up", 28672)], 8192),
                              ("down", [("down", 8192)], 28672)], "down",
                             "Llama-2-70B-shaped decoder block, 4 GEMVs in sequence (q/k/v and gate/up share "
                             "their input and are packed row-wise into one blob each)"),
}
PAPER_CONTEXT = ("paper Table IV: GPTQT 3-bit is 1.24x faster than GPTQ 3-bit (and 3.4x faster than fp16) on "
                 "opt-30b, batch 1, NVIDIA RTX A5000, 128-token generation; no per-GEMV time or GB/s is published")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="opt30b")
    ap.add_argument("--q", type=int, choices=(2, 3), default=3, help="number of sign planes")
    ap.add_argument("--rowwise", action="store_true",
                    help="one scaling group per row (group = N, the paper's setting) instead of groups of 128")
    ap.add_argument("--offset", action="store_true", help="add the per-group fp16 offset term (N(0, 0.01))")
    ap.add_argument("--outliers", action="store_true", help="scale 1 %% of the activation channels by 20")
    ap.add_argument("--batch", type=int, default=1,
                    help="activation vectors per call: 1 = bcq_gemv (the headline), 2..64 = bcq_gemm_skinny")
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

    if not 1 <= args.batch <= 64:
        print("bench.py: --batch must be 1..64", file=sys.stderr)
        sys.exit(2)
    B = args.batch
    LAUNCHES, DOMINANT, WORKLOAD_TEXT = WORKLOADS[args.workload]
    LAYERS = [(name, sum(rows for _, rows in parts), N) for name, parts, N in LAUNCHES]
    Q = args.q

    # ---- build and pack the layer set (not timed) ------------------------------
    layers = {}
    total_bytes = 0
    for name, parts, N in LAUNCHES:
        M = sum(rows for _, rows in parts)
        group = N if args.rowwise else GROUP
        pl = bcq.PackedLayer(M, N, Q, group, args.offset, max_batch=B)
        subs, row0, nbytes = [], 0, 0
        for k, (pname, rows) in enumerate(parts):  # each projection from its own tensors
            L = bcq_synth.make_layer(rows, N, Q, group=group, offset=args.offset, batch=B, seed=k,
                                     outlier_frac=0.01 if args.outliers else 0.0)
            codes = to_dev(L.codes())
            alpha = to_dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16)
            off = to_dev(L.offset.view(np.uint16).astype(np.int16)).view(torch.float16) if args.offset else None
            pl.pack_rows_from(row0, codes, alpha, off)
            torch.cuda.synchronize()
            del codes, alpha, off
            subs.append((row0, L))
            row0 += rows
            nbytes += L.weight_bytes()
        x = to_dev(subs[0][1].x.view(np.uint16).astype(np.int16)).view(torch.float16)  # [B][N]
        y = torch.empty((B, M), dtype=torch.float16, device=dev)
        layers[name] = dict(subs=subs, pl=pl, x=x, y=y, bytes=nbytes, copies=[pl.packed])
        total_bytes += nbytes
    # enough copies that the largest layer alone rotates over at least 1 GiB (13 for 86.7 MB)
    n_copies = max(2, math.ceil(2 ** 30 / max(ent["bytes"] for ent in layers.values())))
    for name in layers:
        ent = layers[name]
        ent["copies"] += [ent["pl"].packed.clone() for _ in range(n_copies - 1)]
    torch.cuda.synchronize()

    def launch(name, i):
        ent = layers[name]
        pl = ent["pl"]
        ws = pl.workspace if pl.workspace_bytes else None
        if B == 1:
            bcq.gemv(pl.desc, ent["copies"][i % n_copies], ent["x"], ent["y"], ws)
        else:
            bcq.gemm_skinny(pl.desc, ent["copies"][i % n_copies], ent["x"], ent["x"].stride(0), ent["y"],
                            ent["y"].stride(0), B, ws)

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

    # ---- the dominant launch, one event pair per launch: median / min over 200 launches after 20 -----
    def per_launch_us(fn, n, warm):
        with torch.cuda.stream(stream):
            for i in range(warm):
                fn(i)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            stream.synchronize()
            for i, (a, b) in enumerate(evs):  # the host runs ahead of the GPU, so the pairs do not see its latency
                a.record(stream)
                fn(warm + i)
                b.record(stream)
            stream.synchronize()
        return sorted(a.elapsed_time(b) * 1e3 for a, b in evs)

    cold = per_launch_us(lambda i: launch(DOMINANT, i), 200, 20)
    copies = layers[DOMINANT]["copies"]
    layers[DOMINANT]["copies"] = copies[:1]  # warm: the same blob every time (L2 / memory-side cache may serve it)
    n_copies_saved, n_copies = n_copies, 1
    warm = per_launch_us(lambda i: launch(DOMINANT, i), 200, 20)
    layers[DOMINANT]["copies"], n_copies = copies, n_copies_saved
    act_bytes = 2 * B * (dom["M"] + dom["N"])
    launch_stats = dict(launches=200, warmup=20, median_us=round(cold[100], 3), min_us=round(cold[0], 3),
                        weight_GBps_at_median=round(dom["weight_bytes"] / cold[100] / 1e3, 1),
                        weights_plus_activations_GBps_at_median=round((dom["weight_bytes"] + act_bytes) / cold[100] / 1e3, 1),
                        warm_single_blob_median_us=round(warm[100], 3),
                        note="hipEvent pair around each eager launch of the dominant layer; cold = rotating weight "
                             "copies, warm = one copy (not an HBM figure)")
    # what a kernel that only reads the same bytes reaches (bcq_read_probe on the dominant layer's blobs)
    sink = torch.empty(bcq.binding.read_probe_sink_bytes(), dtype=torch.uint8, device=dev)
    dom_ent = layers[DOMINANT]
    nbytes_blob = dom_ent["pl"].packed.numel()
    t = timed(lambda i: bcq.read_probe(dom_ent["copies"][i % n_copies], nbytes_blob, sink), args.steps, args.warmup + 2)
    probe_us = t / args.steps * 1e6
    read_probe = dict(bytes=nbytes_blob, us=round(probe_us, 3), GBps=round(nbytes_blob / probe_us / 1e3, 1),
                      what="plain streaming read of the dominant layer's packed weights (no arithmetic)")
    achieved = dom["weight_bytes"] / (dom["us_per_gemv"] * 1e-6) / 1e9
    MFMA_PEAK_TFLOPS = 2500.0  # dense binary16 matrix-core peak
    if B > 1:
        # The single-pass skinny kernel reads the weights once (HBM) and contracts on the matrix cores
        # (binary16 in, fp32 accumulate; useful work 2 * q * M * N * batch flop per launch).  Both roofs are
        # evaluated; the one that needs more time at its peak binds, and `frac` is taken against it.
        flop = 2.0 * Q * dom["M"] * dom["N"] * B
        us = dom["us_per_gemv"]
        t_hbm_us = dom["weight_bytes"] / (HBM_PEAK_GBS * 1e9) * 1e6
        t_mfma_us = flop / (MFMA_PEAK_TFLOPS * 1e12) * 1e6
        tfl = flop / (us * 1e-6) / 1e12
        hbm = dict(bound="hbm", achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                   frac=round(achieved / HBM_PEAK_GBS, 4), time_at_peak_us=round(t_hbm_us, 2))
        mfma = dict(bound="mfma", achieved=round(tfl, 2), peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(tfl / MFMA_PEAK_TFLOPS, 4), time_at_peak_us=round(t_mfma_us, 2))
        binding, other = (hbm, mfma) if t_hbm_us >= t_mfma_us else (mfma, hbm)
        roofline = dict(binding)
        roofline.update(kernel="bcq_gemm_skinny's kernel for the shape (q=%d, %s, %s, batch %d) on %dx%d"
                               % (Q, "offset" if args.offset else "no offset",
                                  "row-wise scales" if args.rowwise else "group 128", B, dom["M"], dom["N"]),
                        bytes_per_launch=dom["weight_bytes"], flop_per_launch=flop, us_per_launch=us, traffic=None,
                        secondary=other)
    else:
        roofline = dict(bound="hbm",
                        kernel="bcq_gemv_kernel (q=%d, %s, %s) on %dx%d"
                               % (Q, "offset" if args.offset else "no offset",
                                  "row-wise scales" if args.rowwise else "group 128", dom["M"], dom["N"]),
                        achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(achieved / HBM_PEAK_GBS, 4), bytes_per_launch=dom["weight_bytes"],
                        us_per_launch=dom["us_per_gemv"], traffic=None)
    # HBM bytes per launch come from two separate rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) whose summary is
    # committed under profiles/; this run does not measure them, and the line says so.
    traffic_file = os.path.join(ROOT, "profiles", "bcq_gemv_opt30b_q3_hbm_traffic.md")
    if os.path.exists(traffic_file) and args.workload == "opt30b" and Q == 3 and B == 1 and not args.offset and not args.rowwise:
        for line in open(traffic_file):
            if line.startswith("hbm_bytes_per_launch_fc2"):
                roofline["traffic"] = float(line.split("=")[1])
                roofline["traffic_source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary in "
                                              "profiles/bcq_gemv_opt30b_q3_hbm_traffic.md (separate runs of this "
                                              "command), not measured by this run")

    # ---- oracle on the host cores, same layer set --------------------------------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import ref
        t0 = time.perf_counter()
        worst = 0.0
        for name, M, N in LAYERS:
            x0 = layers[name]["subs"][0][1].x  # the activations every part of this launch was given
            y_all = layers[name]["y"].cpu().numpy().astype(np.float64)
            for row0, L in layers[name]["subs"]:
                y_ref = ref.gemm(L.planes, L.alpha, L.offset, x0)
                y_gpu = y_all[:, row0:row0 + L.M]
                rms = math.sqrt(float(np.mean(y_ref ** 2)))
                err = np.abs(y_gpu - y_ref) / np.maximum(np.abs(y_ref), rms / 64.0)
                worst = max(worst, float(err.max()))
        t_cpu = time.perf_counter() - t0
        # the two phases of the definition, timed separately on the smallest layer, all threads and one thread
        small = min(LAYERS, key=lambda l: l[1] * l[2])[0]
        Ls = layers[small]["subs"][0][1]
        threads = ref.num_threads()
        phases = {}
        for nthr in (threads, 1):
            ref.set_num_threads(nthr)
            t1 = time.perf_counter()
            W = ref.dequant(Ls.planes, Ls.alpha, Ls.offset)
            t2 = time.perf_counter()
            ref.dense_matmul(W, Ls.x)
            t3 = time.perf_counter()
            phases["threads_%d" % nthr] = dict(dequant_s=round(t2 - t1, 3), matvec_s=round(t3 - t2, 3))
            del W
        ref.set_num_threads(threads)
        cpu = dict(value=round(total_bytes / t_cpu / 1e9, 4), unit="GB/s", cores=threads, kind="oracle",
                   sample="full layer set, one pass (all rows of every layer), fp64 dequant + matvec",
                   seconds=round(t_cpu, 2), phases_on=("%s %dx%d" % (small, Ls.M, Ls.N)), phases=phases)
        parity = dict(max_gated_rel_err=worst, tolerance=2e-3)

    out = {
        "metric": "effective weight GB/s (and us per GEMV), %d-bit batch-%d binary-coding GEMV" % (Q, B),
        "value": round(value_gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 activations, 1-bit planes x%d, f32 accumulate" % Q, "data": "synthetic",
        "config": {"workload": "%s, q=%d, %s%s%s, batch=%d, cold weights (%d rotating copies)"
                               % (WORKLOAD_TEXT, Q, "row-wise scales (group=N)" if args.rowwise else "group=128",
                                  ", with offset" if args.offset else "",
                                  ", outlier channels" if args.outliers else "", B, n_copies), "launches_per_step": len(LAYERS),
                   "weight_bytes_per_step": total_bytes, "launch": "graph" if not args.no_graph else "eager"},
        "pct_of_hbm_peak": round(value_gbs / HBM_PEAK_GBS * 100, 2),
        "layers": per_layer, "roofline": roofline, "launch_stats": launch_stats, "read_probe": read_probe, "cpu_baseline": cpu, "parity": parity,
        "context": PAPER_CONTEXT,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
