"""GPU parity of bcq_from_linear (Sec. II-B Eq. 6, Sec. II-D Eq. 9-11) against oracle/fuse.py:
plane codes and the binary16 fused scales must match bit for bit, and the packed result must
reproduce the product with the dequantised linear weights S * W_q + qbias."""
import numpy as np
import pytest
import torch

import bcq_synth
import paper_2407_02891_amd as bcq
from oracle import fuse, ref
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _labels(partition, n):
    lab = [None] * n
    for c, cls in enumerate(partition):
        for i in cls:
            lab[i - 1] = c
    return lab


def _case(M, N, group, n, partition, seed):
    rng = np.random.default_rng(seed)
    q = len(partition)
    G = N // group
    W_int = rng.integers(0, 2 ** n, size=(M, N), dtype=np.int64)
    W_int[0, : 2 ** n] = np.arange(2 ** n)                       # every integer occurs, ties included
    S = (0.002 + 0.02 * rng.random((M, G))).astype(np.float32)
    qbias = (rng.standard_normal((M, G)) * 0.05).astype(np.float32)
    # oracle: Eq. 6 then Eq. 11, in fp64
    W_q = fuse.nearest_bcchoice(W_int, fuse.bcchoice(partition, n))
    planes, alpha64, z64 = fuse.fuse(W_q, S.astype(np.float64), qbias.astype(np.float64), partition, n, group)
    # device
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    codes = torch.empty((M, N), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((M, G, q), dtype=torch.float16, device="cuda")
    off = torch.empty((M, G), dtype=torch.float16, device="cuda")
    bcq.from_linear(M, N, group, n, q, _labels(partition, n), dev(W_int.astype(np.uint8)), dev(S), dev(qbias),
                    codes, alpha, off)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), bcq_synth.planes_to_codes(planes))
    a16, z16 = alpha64.astype(np.float16), z64.astype(np.float16)  # one rounding from binary64
    assert np.array_equal(alpha.cpu().numpy().view(np.uint16), a16.view(np.uint16))
    assert np.array_equal(off.cpu().numpy().view(np.uint16), z16.view(np.uint16))
    # through the hot path: pack and multiply
    x = rng.standard_normal((1, N)).astype(np.float16)
    pl = bcq.PackedLayer(M, N, q, group, True)
    pl.pack_from(codes, alpha, off)
    y = U.gpu_gemv(pl, U.to_dev(x.view(np.uint16).astype(np.int16)).view(torch.float16))
    U.gate(y[None, :], ref.gemm(planes, a16, z16, x), f"from_linear n={n} {partition}")
    # and against the linear-quantised weights themselves (binary16 scales cost about 2^-11 each)
    W_hat = np.repeat(S.astype(np.float64), group, axis=1) * W_q + np.repeat(qbias.astype(np.float64), group, axis=1)
    y_lin = W_hat @ x[0].astype(np.float64)
    rms = np.sqrt(np.mean(y_lin ** 2))
    assert np.abs(y.astype(np.float64) - y_lin).max() <= 4e-3 * max(rms, np.abs(y_lin).max())


@pytest.mark.parametrize("n,partition", [(3, ((1,), (2, 3))),            # the paper's Eq. 10
                                          (3, ((1, 2), (3,))),
                                          (4, ((1, 2), (3,), (4,))),
                                          (5, ((1, 4), (2, 5), (3,))),
                                          (5, ((1,), (2,), (3, 4, 5))),
                                          (4, ((1,), (2,), (3,), (4,))),  # no tying: plain linear -> 4 planes
                                          (2, ((1, 2),))])               # one plane
def test_from_linear_matches_oracle(n, partition):
    _case(70, 1536, 128, n, partition, seed=n * 10 + len(partition))


def test_from_linear_all_partitions_n5_q3_small_groups():
    """All 25 tyings of 5 planes into 3 classes, groups of 64 columns."""
    for k, partition in enumerate(fuse.all_partitions(5, 3)):
        _case(33, 1024, 64, 5, partition, seed=100 + k)
