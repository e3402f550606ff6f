"""Per-wave timeline of the batch-1 GEMV and of the skinny GEMM's table kernel (diagnostic).

Runs the tracing build of the kernel (libbcq_trace.so: bcq_gemv.hip compiled with -DBCQ_TRACE, built by
`python -m paper_2407_02891_amd.build --trace`) once on a synthetic layer with cold weights and prints, over
all waves of the grid, when each wave reached the fixed points of the kernel and how its time in the tile
loop splits up.  Times are in microseconds since the first wave started (100 MHz real-time counter, 10 ns
steps).  The traced kernel is the product kernel plus the time stamps; it runs a few percent slower.

    python -m paper_2407_02891_amd.trace_gemv --rows 7168 --cols 28672 --q 3

Slots written per wave: 0 wave started, 1 first loads issued, 2 activations (and, unless the early start-up
is used, the first tile) arrived, 3 own share of the tables written, 4 tables complete (barrier passed),
5 first tile in registers, 6 tile loop left, 7 last atomic returned / last store acknowledged; sums over the
wave's tiles: 8 waiting at the top of the loop, 9 completing rows and issuing the atomic, 10 issuing the
next tile's loads (stalls there when the memory pipeline is full), 11 look-ups and scaling, 12 cross-lane
sum; 15 number of tiles.

With --batch B (2..16) the skinny GEMM's table kernel is traced instead:

    python -m paper_2407_02891_amd.trace_gemv --rows 7168 --cols 28672 --q 3 --batch 16

Slots: 0 wave started, 1 first X slice staged and sign table built, 2 last work unit done, 3 last flush done;
sums over the wave's units (one unit = one 32-row tile times one 512-column slice): 12 issuing the requests for
the next unit's tile and X slice, 8 from there until this unit's tile has arrived and is transposed, 9 the 16
MFMA steps with their table and X reads, 10 storing the next X slice to LDS (waits for it), 11 waiting at the
workgroup barrier; 15 number of units.
"""
import argparse
import ctypes
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
TRACE_LIB = os.path.join(HERE, "libbcq_trace.so")
SLOTS = 16
POINTS = [(0, "wave started"), (1, "first loads issued"), (2, "activations arrived"), (3, "own table share written"),
          (4, "tables complete (barrier)"), (5, "first tile in registers"), (6, "tile loop left"),
          (7, "last atomic / store done")]
SUMS = [(8, "waiting for tile + old atomic"), (9, "complete rows + issue atomic"), (10, "issue next tile's loads"),
        (11, "look-ups and scaling"), (12, "cross-lane sum")]


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--rows", type=int, default=7168)
    ap.add_argument("--cols", type=int, default=28672)
    ap.add_argument("--q", type=int, default=3)
    ap.add_argument("--group", type=int, default=128)
    ap.add_argument("--offset", action="store_true")
    ap.add_argument("--workgroups", type=int, default=0, help="0 = automatic")
    ap.add_argument("--waves", type=int, default=0, choices=(0, 4, 8), help="0 = automatic")
    ap.add_argument("--early", type=int, default=0, choices=(0, 1, 2), help="1 = early table build, 2 = never, 0 = automatic")
    ap.add_argument("--batch", type=int, default=1, help="2..16: trace the skinny GEMM's table kernel instead")
    ap.add_argument("--repeats", type=int, default=5, help="traced launches (each on another cold copy); the median launch is reported")
    a = ap.parse_args()

    import numpy as np
    import torch

    import bcq_synth
    import paper_2407_02891_amd as bcq

    if not os.path.exists(TRACE_LIB):
        raise SystemExit(f"{TRACE_LIB} is missing: run `python -m paper_2407_02891_amd.build --trace`")
    T = ctypes.CDLL(TRACE_LIB)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    T.bcq_gemv_trace_shape.restype = i32
    T.bcq_gemv_trace_shape.argtypes = [ctypes.POINTER(bcq.Desc), i32, i32, i32] + [ctypes.POINTER(i32)] * 3
    T.bcq_gemv_trace.restype = i32
    T.bcq_gemv_trace.argtypes = [ctypes.POINTER(bcq.Desc), vp, vp, vp, vp, vp, i32, i32, i32, vp]

    L = bcq_synth.make_layer(a.rows, a.cols, a.q, group=a.group, offset=a.offset, seed=0)
    pl = bcq.PackedLayer(L.M, L.N, L.q, L.group, a.offset, max_batch=max(1, a.batch))

    def dev(arr):
        return torch.from_numpy(np.ascontiguousarray(arr)).cuda()

    pl.pack_from(dev(L.codes()), dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16),
                 dev(L.offset.view(np.uint16).astype(np.int16)).view(torch.float16) if a.offset else None)
    if a.batch > 1:
        return trace_skinny(a, T, L, pl, dev)
    x = dev(L.x.view(np.uint16).astype(np.int16)).view(torch.float16)[0].contiguous()
    y = torch.empty(L.M, dtype=torch.float16, device="cuda")
    y_ref = pl.gemv(x).clone()
    # enough copies of the blob that a launch never finds its weights in the caches
    copies = [pl.packed] + [pl.packed.clone() for _ in range(max(2, (1 << 30) // pl.packed.numel()))]
    wg, nw, early = i32(), i32(), i32()
    T.bcq_gemv_trace_shape(ctypes.byref(pl.desc), a.workgroups, a.waves, a.early, ctypes.byref(wg), ctypes.byref(nw), ctypes.byref(early))
    nwaves = wg.value * nw.value
    trace = torch.zeros(nwaves * SLOTS, dtype=torch.int32, device="cuda")
    ws = pl.workspace.data_ptr() if pl.workspace_bytes else None
    stream = torch.cuda.current_stream().cuda_stream
    runs = []
    for rep in range(a.repeats + 2):
        blob = copies[(rep + 1) % len(copies)]
        trace.zero_()
        torch.cuda.synchronize()
        rc = T.bcq_gemv_trace(ctypes.byref(pl.desc), blob.data_ptr(), x.data_ptr(), y.data_ptr(), ws, trace.data_ptr(),
                              a.workgroups, a.waves, a.early, stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), "the traced kernel must give the product kernel's result"
        if rep >= 2:  # the first two launches warm up clocks and translation caches
            t = trace.cpu().numpy().astype(np.int64).reshape(nwaves, SLOTS) & 0xffffffff
            runs.append(t)
    runs.sort(key=lambda t: (t[:, 7].max() - t[:, 0].min()))
    t = runs[len(runs) // 2]
    t0 = t[:, 0].min()
    print(f"layer {a.rows}x{a.cols} q={a.q} group={a.group}{' offset' if a.offset else ''}: {wg.value} workgroups x {nw.value} waves, "
          f"early table build {'on' if early.value else 'off'}; weights {L.weight_bytes()} B; "
          f"median of {a.repeats} traced launches by length; kernel {0.01 * (t[:, 7].max() - t0):.2f} us from first wave start to last wave end")
    print(f"{'point (us since first wave start)':38s} {'min':>7s} {'p10':>7s} {'median':>7s} {'p90':>7s} {'max':>7s}")
    work = t[:, 15] > 0
    for slot, name in POINTS:
        sel = work if slot in (5,) else np.ones(nwaves, dtype=bool)
        v = np.sort((t[sel, slot] - t0) * 0.01)
        print(f"{name:38s} {v[0]:7.2f} {v[len(v) // 10]:7.2f} {v[len(v) // 2]:7.2f} {v[len(v) * 9 // 10]:7.2f} {v[-1]:7.2f}")
    print(f"{'time per wave inside the tile loop (us)':38s} {'min':>7s} {'p10':>7s} {'median':>7s} {'p90':>7s} {'max':>7s}")
    for slot, name in SUMS:
        v = np.sort(t[work, slot] * 0.01)
        print(f"{name:38s} {v[0]:7.2f} {v[len(v) // 10]:7.2f} {v[len(v) // 2]:7.2f} {v[len(v) * 9 // 10]:7.2f} {v[-1]:7.2f}")
    tiles = t[:, 15]
    print(f"tiles per wave: min {tiles.min()} max {tiles.max()} mean {tiles.mean():.2f}; waves without a tile: {(tiles == 0).sum()}")
    last = int(np.argmax(t[:, 7]))
    print("the wave that ended last (workgroup %d, wave %d):" % (last // nw.value, last % nw.value),
          " ".join(f"{name.split(' (')[0]} {0.01 * (t[last, slot] - t0):.2f}" for slot, name in POINTS), f"tiles {t[last, 15]}")


def trace_skinny(a, T, L, pl, dev):
    import numpy as np
    import torch
    import paper_2407_02891_amd as bcq
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    T.bcq_skinny_trace.restype = i32
    T.bcq_skinny_trace.argtypes = [ctypes.POINTER(bcq.Desc), vp, vp, i32, vp, i32, i32, vp, vp, i32, i32, vp]
    if not 2 <= a.batch <= 16:
        raise SystemExit("--batch must be 2..16")
    rng = np.random.default_rng(1)
    X = torch.from_numpy(rng.standard_normal((a.batch, L.N)).astype(np.float16)).cuda()
    Y = torch.empty((a.batch, L.M), dtype=torch.float16, device="cuda")
    bcq.set_option("skinny_version", 2)
    if a.waves:
        bcq.set_option("waves", a.waves)
    Y_ref = pl.gemm_skinny(X).clone()
    copies = [pl.packed] + [pl.packed.clone() for _ in range(max(2, (1 << 30) // pl.packed.numel()))]
    cap = 2048  # workgroups the trace buffer has room for (8 records each)
    trace = torch.zeros(cap * 8 * SLOTS, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    runs = []
    for rep in range(a.repeats + 2):
        blob = copies[(rep + 1) % len(copies)]
        trace.zero_()
        torch.cuda.synchronize()
        rc = T.bcq_skinny_trace(ctypes.byref(pl.desc), blob.data_ptr(), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0),
                                a.batch, pl.workspace.data_ptr(), trace.data_ptr(), cap, a.waves, stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_ref), "the traced kernel must give the product kernel's result"
        if rep >= 2:
            t = trace.cpu().numpy().astype(np.int64).reshape(cap * 8, SLOTS) & 0xffffffff
            runs.append(t[t[:, 15] > 0])
    runs.sort(key=lambda t: (t[:, 3].max() - t[:, 0].min()))
    t = runs[len(runs) // 2]
    t0 = t[:, 0].min()
    print(f"layer {a.rows}x{a.cols} q={a.q} group={a.group}{' offset' if a.offset else ''} batch {a.batch}: {len(t)} waves with work; "
          f"weights {L.weight_bytes()} B; median of {a.repeats} traced launches by length; "
          f"kernel {0.01 * (t[:, 3].max() - t0):.2f} us from first wave start to last wave end")
    print(f"{'point (us since first wave start)':38s} {'min':>7s} {'p10':>7s} {'median':>7s} {'p90':>7s} {'max':>7s}")
    for slot, name in [(0, "wave started"), (1, "X staged, sign table built"), (2, "last unit done"), (3, "last flush done")]:
        v = np.sort((t[:, slot] - t0) * 0.01)
        print(f"{name:38s} {v[0]:7.2f} {v[len(v) // 10]:7.2f} {v[len(v) // 2]:7.2f} {v[len(v) * 9 // 10]:7.2f} {v[-1]:7.2f}")
    print(f"{'time per wave over its units (us)':38s} {'min':>7s} {'p10':>7s} {'median':>7s} {'p90':>7s} {'max':>7s}")
    for slot, name in [(12, "issue requests for the next unit"), (8, "wait for tile + transpose"), (9, "16 MFMA steps (table + X reads)"),
                       (10, "store next X slice (waits for it)"), (11, "barrier")]:
        v = np.sort(t[:, slot] * 0.01)
        print(f"{name:38s} {v[0]:7.2f} {v[len(v) // 10]:7.2f} {v[len(v) // 2]:7.2f} {v[len(v) * 9 // 10]:7.2f} {v[-1]:7.2f}")
    units = t[:, 15]
    print(f"units per wave: min {units.min()} max {units.max()} mean {units.mean():.2f}")
    per_unit = (t[:, 8] + t[:, 9] + t[:, 10] + t[:, 11] + t[:, 12]) * 0.01 / units
    print(f"time per unit: median {np.median(per_unit):.2f} us; of which MFMA steps {np.median(t[:, 9] * 0.01 / units):.2f} us")


if __name__ == "__main__":
    main()
