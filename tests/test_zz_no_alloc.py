"""bcq_gemv_noalloc (the entry point for callers that cannot allocate: its split-K accumulators live in a
static device array inside the library) against bcq_gemv, through the C ABI: two calls in a row, the second
on a smaller layer, each bit for bit equal to bcq_gemv's result and within the parity gate of the oracle."""
import numpy as np
import pytest
import torch

import bcq_synth
import paper_2407_02891_amd as bcq
from oracle import ref
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def test_noalloc_matches_gemv_on_two_calls_in_a_row():
    big = bcq_synth.make_layer(1500, 4096, 3, group=128, offset=True, seed=71)      # 47 row tiles (ragged), 8 slices
    small = bcq_synth.make_layer(200, 1536, 2, group=128, offset=False, seed=72)    # fewer rows and slices
    outs = []
    for L in (big, small):
        pl = U.upload_and_pack(L)
        x = U.x_dev(L)[0].contiguous()
        y_ws = torch.empty(L.M, dtype=torch.float16, device="cuda")
        bcq.gemv(pl.desc, pl.packed, x, y_ws, pl.workspace)
        outs.append((L, pl, x, y_ws))
    torch.cuda.synchronize()
    got = []
    for L, pl, x, y_ws in outs:                      # back to back, no synchronisation in between
        y = torch.full((L.M,), 7.0, dtype=torch.float16, device="cuda")
        bcq.gemv_noalloc(pl.desc, pl.packed, x, y)
        got.append(y)
    torch.cuda.synchronize()
    for (L, pl, x, y_ws), y in zip(outs, got):
        assert torch.equal(y, y_ws), f"{L.M}x{L.N}: differs from bcq_gemv"
        U.gate(y.cpu().numpy()[None, :], ref.gemm(L.planes, L.alpha, L.offset, L.x), f"noalloc {L.M}x{L.N}")
    # and once more on the large layer after the small one: the array is shared and cleared per call
    L, pl, x, y_ws = outs[0]
    y = torch.zeros(L.M, dtype=torch.float16, device="cuda")
    bcq.gemv_noalloc(pl.desc, pl.packed, x, y)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ws)


def test_noalloc_single_slice_and_refusal():
    L = bcq_synth.make_layer(70, 512, 3, group=128, offset=False, seed=73)          # one column slice: no split-K
    pl = U.upload_and_pack(L)
    x = U.x_dev(L)[0].contiguous()
    y = torch.empty(L.M, dtype=torch.float16, device="cuda")
    bcq.gemv_noalloc(pl.desc, pl.packed, x, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().view(np.uint16), U.gpu_gemv(pl, x).view(np.uint16))
    # more rows than the static array holds: refused on the host, nothing launched
    d = bcq.Desc(bcq.binding.BCQ_NOALLOC_MAX_ROWS + 1, 1024, 1, 128, 0, bcq.binding.BCQ_LAYOUT_VERSION)
    with pytest.raises(bcq.BcqError) as e:
        bcq.gemv_noalloc(d, pl.packed, x, y)
    assert e.value.status == bcq.binding.BCQ_ERR_SCRATCH_LIMIT
