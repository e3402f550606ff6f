"""Helpers for the GPU parity tests: upload a synthetic layer, run it through
the C ABI (via the binding), and compare with the fp64 oracle."""
import numpy as np
import torch

import paper_2407_02891_amd as bcq
from oracle import ref

# Tolerance of the parity gate.  The target states "max relative error 2e-3
# (fp32 accumulate)"; a per-element relative error is unbounded where y
# cancels to ~0, so an element is compared against max(|y_ref|, rms(y_ref)/64).
RTOL = 2e-3
FLOOR_DIV = 64.0


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_and_pack(L, max_batch=1):
    """Layer (bcq_synth.Layer) -> PackedLayer on the GPU (bcq_pack)."""
    pl = bcq.PackedLayer(L.M, L.N, L.q, L.group, L.offset is not None, max_batch=max_batch)
    codes = to_dev(L.codes())
    alpha = to_dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16)
    off = None if L.offset is None else to_dev(L.offset.view(np.uint16).astype(np.int16)).view(torch.float16)
    pl.pack_from(codes, alpha, off)
    torch.cuda.synchronize()
    return pl


def x_dev(L):
    return to_dev(L.x.view(np.uint16).astype(np.int16)).view(torch.float16)


def gpu_gemv(pl, xd):
    y = pl.gemv(xd[0] if xd.dim() == 2 else xd)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_gemm(pl, Xd):
    Y = pl.gemm_skinny(Xd)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


def gate(y_gpu16, y_ref, what=""):
    """Assert the parity gate; returns (max gated error ratio, normwise error)."""
    y_gpu = y_gpu16.astype(np.float64)
    assert y_gpu.shape == y_ref.shape, (y_gpu.shape, y_ref.shape)
    assert np.all(np.isfinite(y_gpu)), what
    rms = np.sqrt(np.mean(y_ref ** 2))
    denom = np.maximum(np.abs(y_ref), rms / FLOOR_DIV)
    ratio = np.abs(y_gpu - y_ref) / np.where(denom > 0, denom, 1.0)
    if rms == 0:
        assert np.array_equal(y_gpu, y_ref), what
        return 0.0, 0.0
    worst = float(ratio.max())
    assert worst <= RTOL, f"{what}: gated rel err {worst:.3e} > {RTOL} at {np.unravel_index(ratio.argmax(), ratio.shape)}"
    return worst, float(np.abs(y_gpu - y_ref).max() / np.abs(y_ref).max())


def oracle_rows(L, rows):
    """Oracle result for a subset of rows (each output row depends only on its
    own planes/alpha/offset row, so the sub-layer is evaluated as is)."""
    rows = np.asarray(rows)
    planes = np.ascontiguousarray(L.planes[:, rows])
    alpha = np.ascontiguousarray(L.alpha[rows])
    off = None if L.offset is None else np.ascontiguousarray(L.offset[rows])
    return ref.gemm(planes, alpha, off, L.x)
