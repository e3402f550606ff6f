"""GPU parity at the benchmark's full layer sizes, in the launch configuration
bench.py times (automatic row split).  The oracle evaluates a sample of rows
(first and last row tiles plus random rows) one by one."""
import numpy as np
import pytest

import bcq_synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _sample_rows(M, n=192, seed=0):
    rng = np.random.default_rng(seed)
    rows = set(range(0, 32)) | set(range(M - 32, M)) | set(rng.choice(M, size=min(n, M), replace=False).tolist())
    return np.array(sorted(rows))


def _check(M, N, q, offset, batch=1, **kw):
    L = bcq_synth.make_layer(M, N, q, group=128, offset=offset, batch=batch, seed=0, **kw)
    pl = U.upload_and_pack(L, max_batch=batch)
    xd = U.x_dev(L)
    y = U.gpu_gemv(pl, xd)[None, :] if batch == 1 else U.gpu_gemm(pl, xd)
    rows = _sample_rows(M)
    y_ref = U.oracle_rows(L, rows)
    worst, normwise = U.gate(y[:, rows], y_ref, f"{M}x{N} q={q} z={offset} b={batch}")
    print(f"{M}x{N} q={q} z={offset} b={batch}: gated {worst:.2e} normwise {normwise:.2e}")


@pytest.mark.parametrize("M,N", [(7168, 7168), (28672, 7168), (7168, 28672)])
def test_opt30b_q3(M, N):
    """configs[1]"""
    _check(M, N, 3, False)


@pytest.mark.parametrize("M,N", [(7168, 7168), (28672, 7168), (7168, 28672)])
def test_opt30b_q2_offset(M, N):
    """configs[2], batch 1"""
    _check(M, N, 2, True)


@pytest.mark.parametrize("M,N", [(9216, 9216), (36864, 9216), (9216, 36864)])
def test_opt66b_q3_outliers(M, N):
    """configs[3], batch 1"""
    _check(M, N, 3, False, outlier_frac=0.01)


@pytest.mark.parametrize("q", [2, 3])
@pytest.mark.parametrize("M,N", [(8192, 8192), (1024, 8192), (28672, 8192), (8192, 28672)])
def test_llama70b_shapes(M, N, q):
    """configs[4], each distinct shape on its own: q/o, k/v (GQA), gate/up, down; q = 2 and 3"""
    _check(M, N, q, False)


@pytest.mark.parametrize("M,N,q,offset,batch", [(7168, 7168, 2, True, 8), (28672, 7168, 2, True, 8),
                                                  (7168, 28672, 2, True, 8),
                                                  (9216, 9216, 3, False, 4), (9216, 9216, 3, False, 16),
                                                  (36864, 9216, 3, False, 4), (36864, 9216, 3, False, 16),
                                                  (9216, 36864, 3, False, 4), (9216, 36864, 3, False, 16),
                                                  (7168, 28672, 3, False, 64),
                                                  (7168, 28672, 3, False, 32), (7168, 7168, 2, True, 24),
                                                  (7168, 28672, 3, False, 2), (9216, 36864, 3, True, 2)])
def test_skinny_fullsize(M, N, q, offset, batch):
    """configs[2] (q=2 with offset, batch 8, all three layers), configs[3] (batch 4 and 16, outlier channels,
    all three layers), the dominant layer of configs[1] at the widest batch of one pass (64), 17..32 columns
    (the table kernel with two column groups, which large layers use), and two vectors (the two-vector table
    kernel, in the launch shape large layers get)"""
    _check(M, N, q, offset, batch=batch, outlier_frac=0.01 if 9216 in (M, N) else 0.0)


@pytest.mark.parametrize("q", [2, 3])
def test_llama70b_block_in_sequence(q):
    """configs[4]: the seven GEMVs of the decoder block (q, k, v, o, gate, up, down) enqueued back to back on
    one stream with ONE shared workspace and no synchronisation in between; every output is then checked
    on sampled rows.  (The workspace is left zero by each call, which is what lets the next one use it.)"""
    import torch
    import paper_2407_02891_amd as bcq
    layers = []
    ws_bytes = 0
    for k, (name, M, N) in enumerate(bcq_synth.LLAMA2_70B_BLOCK):
        L = bcq_synth.make_layer(M, N, q, group=128, offset=False, seed=k)
        pl = U.upload_and_pack(L)
        # keep only what the check needs: the sampled rows' operands and the activations
        rows = _sample_rows(M, n=64, seed=k)
        keep = (np.ascontiguousarray(L.planes[:, rows]), np.ascontiguousarray(L.alpha[rows]), L.x.copy())
        layers.append((name, pl, U.x_dev(L)[0].contiguous(), torch.empty(M, dtype=torch.float16, device="cuda"), rows, keep))
        ws_bytes = max(ws_bytes, pl.workspace_bytes)
        del L
    shared = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    bcq.workspace_init(shared)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for rep in range(2):                      # twice: the second pass starts from what the first left behind
            for name, pl, x, y, rows, keep in layers:
                bcq.gemv(pl.desc, pl.packed, x, y, shared)
    stream.synchronize()
    torch.cuda.synchronize()
    from oracle import ref
    for name, pl, x, y, rows, (planes, alpha, xh) in layers:
        U.gate(y.cpu().numpy()[None, rows], ref.gemm(planes, alpha, None, xh), f"block layer {name} q={q}")
    assert not shared.cpu().numpy().any()


def test_llama70b_fused_qkv_equals_three_gemvs():
    """configs[4]: the q, k and v projections (8192, 1024, 1024 rows of 8192 columns) read the
    same activations.  Packed row-wise into one blob (bcq_pack_rows) they run as ONE GEMV whose
    output is, bit for bit, the concatenation of the three separate GEMVs, and matches the oracle."""
    import torch
    import paper_2407_02891_amd as bcq
    N, q = 8192, 3
    parts = [bcq_synth.make_layer(M, N, q, group=128, offset=False, seed=s) for s, M in enumerate((8192, 1024, 1024))]
    xd = U.x_dev(parts[0])
    fused = bcq.PackedLayer(sum(L.M for L in parts), N, q, 128, False)
    row0, separate = 0, []
    for L in parts:
        codes = U.to_dev(L.codes())
        alpha = U.to_dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16)
        fused.pack_rows_from(row0, codes, alpha, None)
        row0 += L.M
        separate.append(U.gpu_gemv(U.upload_and_pack(L), xd))
    y = U.gpu_gemv(fused, xd)
    assert np.array_equal(y.view(np.uint16), np.concatenate(separate).view(np.uint16))
    row0 = 0
    for L in parts:
        rows = _sample_rows(L.M, n=96)
        planes, alpha = np.ascontiguousarray(L.planes[:, rows]), np.ascontiguousarray(L.alpha[rows])
        from oracle import ref
        y_ref = ref.gemm(planes, alpha, None, parts[0].x)
        U.gate(y[None, row0 + rows], y_ref, f"fused qkv part at row {row0}")
        row0 += L.M
