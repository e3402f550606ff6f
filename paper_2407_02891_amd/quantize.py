"""Quantise one linear layer to the packed binary coding with the device quantiser
(paper Sec. II-A Eq. 1-2, Sec. II-B Eq. 5-6, Sec. II-C Eq. 7, Sec. II-D Eq. 11).

`quantize_layer` chains the C-ABI calls: search (scale grid x plane tyings, per row), factorisation
of the inverse dampened Hessian, GPTQ pass, fusion into q sign planes with per-row scales and offset,
packing.  Every step runs in the library's kernels; torch only holds the buffers.

Run as a module for a timed run on a synthetic layer (timings only; the checks of the result
live in tests/test_gpu_quantizer.py):
    python -m paper_2407_02891_amd.quantize --rows 7168 --cols 7168 --bits 3 --planes 2 --grid 8
"""
import argparse
import json
import time

import torch

from . import binding as B


def inverse_hessian_factor(H, damp=0.01):
    """Upper triangular U with (H + damp * mean(diag H) I)^-1 = U^T U, binary32 on H's device."""
    N = H.shape[0]
    U = torch.empty((N, N), dtype=torch.float32, device=H.device)
    ws = torch.empty(B.quant_factor_workspace_bytes(N), dtype=torch.uint8, device=H.device)
    B.quant_factor(N, damp, H, U, ws)
    return U


def quantize_layer(W, H, n_bits, q, grid=8, damp=0.01, timings=None):
    """W [M][N] binary32 and H [N][N] binary32 (2 X X^T) on the GPU -> (PackedLayer, info).
    info holds S, qbias, class_of_plane, search_error, w_int and the factor U as device tensors."""
    M, N = W.shape
    dev = W.device
    S = torch.empty(M, dtype=torch.float32, device=dev)
    qbias = torch.empty(M, dtype=torch.float32, device=dev)
    labels = torch.empty((M, n_bits), dtype=torch.int8, device=dev)
    err = torch.empty(M, dtype=torch.float32, device=dev)
    w_int = torch.empty((M, N), dtype=torch.uint8, device=dev)
    ws = torch.empty(B.quant_workspace_bytes(M, N), dtype=torch.uint8, device=dev)

    def timed(name, fn):
        if timings is None:
            return fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        timings[name] = (time.perf_counter() - t0) * 1e3
        return out

    timed("search_ms", lambda: B.quant_search(M, N, n_bits, q, grid, W, H, S, qbias, labels, err, ws))
    U = timed("factor_ms", lambda: inverse_hessian_factor(H, damp))
    timed("gptq_ms", lambda: B.quant_gptq(M, N, n_bits, q, W, U, S, qbias, labels, w_int, ws))
    codes = torch.empty((M, N), dtype=torch.uint8, device=dev)
    alpha = torch.empty((M, 1, q), dtype=torch.float16, device=dev)
    offset = torch.empty((M, 1), dtype=torch.float16, device=dev)
    layer = B.PackedLayer(M, N, q, N, True)

    def fuse_and_pack():
        B.from_linear_rows(M, N, n_bits, q, labels, w_int, S, qbias, codes, alpha, offset)
        layer.pack_from(codes, alpha, offset)

    timed("fuse_pack_ms", fuse_and_pack)
    return layer, {"S": S, "qbias": qbias, "class_of_plane": labels, "search_error": err, "w_int": w_int, "U": U}


def _main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--rows", type=int, default=7168)
    ap.add_argument("--cols", type=int, default=7168)
    ap.add_argument("--bits", type=int, default=3, help="bits of the intermediate linear quantisation (n)")
    ap.add_argument("--planes", type=int, default=2, help="binary-coding planes (q)")
    ap.add_argument("--grid", type=int, default=8, help="scale candidates inside Eq. 7's interval")
    ap.add_argument("--seed", type=int, default=0)
    a = ap.parse_args()
    M, N = a.rows, a.cols
    g = torch.Generator(device="cuda").manual_seed(a.seed)
    W = torch.randn((M, N), device="cuda", generator=g) * 0.02
    X = torch.randn((N, 2 * N), device="cuda", generator=g) + 0.5 * (
        torch.randn((N, 8), device="cuda", generator=g) @ torch.randn((8, 2 * N), device="cuda", generator=g))
    H = torch.zeros((N, N), dtype=torch.float32, device="cuda")
    Xt = X.T.contiguous()                      # [sample][channel]
    del X
    B.quant_hessian(N, Xt.shape[0], Xt, H)     # H = 2 X X^T (Sec. II-A)
    del Xt
    timings = {}
    layer, info = quantize_layer(W, H, a.bits, a.planes, a.grid, timings=timings)
    tyings = {3: {2: 3, 3: 1}, 4: {2: 7, 3: 6, 4: 1}, 5: {3: 25}}.get(a.bits, {}).get(a.planes)
    out = {"rows": M, "cols": N, "n_bits": a.bits, "q": a.planes, "grid": a.grid, "tyings": tyings,
           **{k: round(v, 2) for k, v in timings.items()}}
    if tyings:
        per = timings["search_ms"] / (a.grid * tyings)
        out["search_ms_per_candidate"] = round(per, 2)
        out["search_tflops_fp32"] = round(2.0 * M * N * N / (per * 1e-3) / 1e12, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    _main()
