"""GPU parity: bcq_pack + bcq_gemv / bcq_gemm_skinny through the C ABI against
the fp64 oracle, element by element, on the same seeded inputs."""
import numpy as np
import pytest
import torch

import bcq_synth
import paper_2407_02891_amd as bcq
from oracle import ref
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _run_case(M, N, q, group, offset, batch=1, seed=0, **kw):
    L = bcq_synth.make_layer(M, N, q, group=group, offset=offset, batch=batch, seed=seed, **kw)
    pl = U.upload_and_pack(L, max_batch=batch)
    xd = U.x_dev(L)
    y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    if batch == 1:
        y = U.gpu_gemv(pl, xd)[None, :]
    else:
        y = U.gpu_gemm(pl, xd)
    return U.gate(y, y_ref, f"M={M} N={N} q={q} g={group} z={offset} b={batch}")


def test_config0_768x768_q3():
    """configs[0]: 768x768, q=3, group 128, no offset, batch 1, seed 0."""
    worst, normwise = _run_case(768, 768, 3, 128, False)
    print(f"config0 gated {worst:.2e} normwise {normwise:.2e}")


@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("offset", [False, True])
def test_planes_and_offset(q, offset):
    _run_case(256, 1536, q, 128, offset, seed=q)


@pytest.mark.parametrize("M,N", [(1, 32), (31, 96), (33, 544), (100, 1120), (257, 2080), (1000, 512), (64, 4096)])
def test_ragged_shapes(M, N):
    """Rows not a multiple of 32, columns not a multiple of 512 (padded tiles),
    single-slice and many-slice cases."""
    group = 128 if N % 128 == 0 else N
    _run_case(M, N, 3, group, True, seed=M)


@pytest.mark.parametrize("group", [128, 256, 512, 2048])
def test_group_sizes_multiple_of_128(group):
    _run_case(96, 2048, 3, group, True, seed=group)
    _run_case(96, 2048, 2, group, False, seed=group + 1)


def test_exact_inputs_bit_for_bit():
    """alpha powers of two, integer x and offset: fp16/fp32/fp64 are all exact,
    so the GPU result must equal the oracle exactly (any difference is an
    indexing error), across slices, ragged edges and split-K."""
    for (M, N, q, off) in [(96, 1536, 3, True), (130, 2592 - 32, 2, False), (64, 512, 3, True), (2048, 1024, 3, False)]:
        group = 128 if N % 128 == 0 else N
        L = bcq_synth.make_exact_layer(M, N, q, group=group, offset=off, seed=M + q)
        pl = U.upload_and_pack(L)
        y = U.gpu_gemv(pl, U.x_dev(L)).astype(np.float64)
        y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)[0]
        assert np.abs(y_ref).max() < 2048, "test inputs must stay exactly representable in fp16"
        assert np.array_equal(y, y_ref), (M, N, q, off, np.abs(y - y_ref).max())


def test_pack_unpack_identity():
    L = bcq_synth.make_layer(100, 1120, 3, group=1120, offset=True, seed=9)
    pl = U.upload_and_pack(L)
    codes = torch.empty((L.M, L.N), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((L.M, 1, L.q), dtype=torch.float16, device="cuda")
    off = torch.empty((L.M, 1), dtype=torch.float16, device="cuda")
    bcq.unpack(pl.desc, pl.packed, codes, alpha, off)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), L.codes())
    assert np.array_equal(alpha.cpu().numpy().view(np.uint16), L.alpha.view(np.uint16))
    assert np.array_equal(off.cpu().numpy().view(np.uint16), L.offset.view(np.uint16))


def test_repeated_calls_are_deterministic_and_workspace_self_resets():
    L = bcq_synth.make_layer(512, 4096, 3, group=128, offset=False, seed=21)
    pl = U.upload_and_pack(L)
    xd = U.x_dev(L)
    first = U.gpu_gemv(pl, xd).view(np.uint16)
    for _ in range(20):
        again = U.gpu_gemv(pl, xd).view(np.uint16)
        assert np.array_equal(first, again)
    assert not pl.workspace.cpu().numpy().any(), "split-K accumulators must be zero again after a call"


def test_grid_size_does_not_change_results():
    L = bcq_synth.make_layer(700, 3072, 3, group=128, offset=True, seed=33)
    pl = U.upload_and_pack(L)
    xd = U.x_dev(L)
    outs = []
    try:
        for split in (1, 2, 5, 37, 200, 0):
            bcq.set_option("workgroups", split)
            outs.append(U.gpu_gemv(pl, xd).view(np.uint16).copy())
    finally:
        bcq.set_option("workgroups", 0)
    for o in outs[1:]:
        assert np.array_equal(outs[0], o)
    U.gate(outs[0].view(np.float16)[None, :], ref.gemm(L.planes, L.alpha, L.offset, L.x))


@pytest.mark.parametrize("early", [1, 2])
@pytest.mark.parametrize("waves", [4, 8])
def test_gemv_early_table_build_and_wave_count_do_not_change_results(early, waves):
    """The GEMV in both start-up orders (tables built before / after the first tile has arrived) and with 4 and
    8 waves per workgroup, forced on shapes that the automatic choice would run otherwise: bit for bit the
    oracle's result on exact inputs (ragged rows and columns, waves without a tile), gate on random ones."""
    try:
        bcq.set_option("gemv_early", early)
        bcq.set_option("waves", waves)
        for (M, N, q, off) in [(70, 1536, 3, True), (1000, 2592 - 32, 2, False), (40, 512, 4, True)]:
            group = 128 if N % 128 == 0 else N
            L = bcq_synth.make_exact_layer(M, N, q, group=group, offset=off, seed=M + q + early)
            y = U.gpu_gemv(U.upload_and_pack(L), U.x_dev(L)).astype(np.float64)
            assert np.array_equal(y, ref.gemm(L.planes, L.alpha, L.offset, L.x)[0]), (M, N, q, off)
        _run_case(600, 4096, 3, 128, True, seed=early + waves)
    finally:
        bcq.set_option("gemv_early", 0)
        bcq.set_option("waves", 0)


def test_subnormal_alpha_and_zero_inputs():
    L = bcq_synth.make_layer(64, 1024, 3, group=128, offset=False, seed=5)
    a = L.alpha.view(np.uint16).copy()
    a[:, :, 2] = 0x0001                      # smallest subnormal in the last plane
    a[:, :, 1] = 0x03FF                      # largest subnormal
    L.alpha = a.view(np.float16)
    pl = U.upload_and_pack(L)
    y = U.gpu_gemv(pl, U.x_dev(L))
    U.gate(y[None, :], ref.gemm(L.planes, L.alpha, None, L.x))
    # all-zero activations give exactly zero
    xz = torch.zeros(L.N, dtype=torch.float16, device="cuda")
    assert not U.gpu_gemv(pl, xz).view(np.uint16).any()


@pytest.mark.parametrize("version", [1, 2])
@pytest.mark.parametrize("batch", [1, 5, 40])
@pytest.mark.parametrize("group,offset", [(128, False), (128, True), (64, False)])
def test_all_subnormal_alpha_is_exact(version, batch, group, offset):
    """Every alpha (and offset) a binary16 subnormal (k * 2^-24, k = 1..1023), x small integers: each
    product and every partial sum is a multiple of 2^-24 below 2^24 of them, hence exact in binary32 and
    binary64 alike, so the result must be the oracle's rounded once to binary16 -- bit for bit.  A path
    that flushed subnormal scales (in a conversion, or as a matrix-core operand in the kernel that folds
    alpha into it) would return zeros (sums of offsets only).  Batch 1 is the table GEMV, 5 and 40 the
    two skinny kernels (groups of 64 always take the alpha-folding one)."""
    L = bcq_synth.make_exact_layer(150, 2048, 3, group=group, offset=offset, batch=batch, seed=90 + batch)
    rng = np.random.default_rng(batch + group)
    L.alpha = rng.integers(1, 1024, size=L.alpha.shape, dtype=np.uint16).view(np.float16)
    assert np.all(L.alpha.astype(np.float64) < 2.0 ** -14) and np.all(L.alpha.astype(np.float64) > 0)
    if offset:  # subnormal offsets of either sign, so that the scales are not drowned by the offset term
        z = rng.integers(1, 1024, size=L.offset.shape, dtype=np.uint16) | (rng.integers(0, 2, size=L.offset.shape, dtype=np.uint16) << 15)
        L.offset = z.view(np.float16)
    y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    assert np.abs(y_ref).max() > 2.0 ** -12, "the scales must matter"
    expect = y_ref.astype(np.float16).astype(np.float64)
    pl = U.upload_and_pack(L, max_batch=batch)
    try:
        bcq.set_option("skinny_version", version)
        Y = U.gpu_gemv(pl, U.x_dev(L))[None, :] if batch == 1 else U.gpu_gemm(pl, U.x_dev(L))
    finally:
        bcq.set_option("skinny_version", 0)
    assert np.array_equal(Y.astype(np.float64), expect), np.abs(Y.astype(np.float64) - expect).max()


def test_gemm_skinny_refuses_a_batch_beyond_the_workspace():
    """PackedLayer sizes its workspace for max_batch; a larger batch must be refused on the host (the kernel
    would address accumulators past the allocation), as must a batch outside 1..BCQ_MAX_BATCH."""
    L = bcq_synth.make_layer(64, 1024, 2, group=128, offset=False, batch=4, seed=1)
    pl = U.upload_and_pack(L, max_batch=2)
    X = U.x_dev(L)
    with pytest.raises(bcq.BcqError) as e:
        pl.gemm_skinny(X)
    assert e.value.status == bcq.binding.BCQ_ERR_WORKSPACE
    Y = U.gpu_gemm(pl, X[:2].contiguous())
    U.gate(Y, ref.gemm(L.planes, L.alpha, None, L.x[:2]))
    big = torch.zeros((bcq.binding.BCQ_MAX_BATCH + 1, L.N), dtype=torch.float16, device="cuda")
    with pytest.raises(bcq.BcqError) as e:
        bcq.PackedLayer(64, 1024, 2, 128, False, max_batch=bcq.binding.BCQ_MAX_BATCH).pack_from(
            U.to_dev(L.codes()), U.to_dev(L.alpha.view(np.uint16).astype(np.int16)).view(torch.float16), None).gemm_skinny(big)
    assert e.value.status == bcq.binding.BCQ_ERR_INVALID_ARG


@pytest.mark.parametrize("shift,ok", [(8, True), (12, True)])
def test_small_outputs_and_the_split_k_quantum(shift, ok):
    """Partial sums cross the column slices as multiples of 2^-34, so a result carries an absolute error of up
    to ceil(N/512) * 2^-35 whatever its size.  With every alpha scaled down by 2^shift (rms(y) ~ 6e-3 and
    4e-4 here, 16 slices) the gate still holds with room: the documented floor is rms(y) >= 1e-6 * ceil(N/512)."""
    L = bcq_synth.make_layer(128, 8192, 3, group=128, offset=False, batch=4, seed=17)
    L.alpha = (L.alpha.astype(np.float32) * 2.0 ** -shift).astype(np.float16)
    y_ref = ref.gemm(L.planes, L.alpha, None, L.x)
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    assert rms >= 1e-6 * 16 * 8, rms
    pl = U.upload_and_pack(L, max_batch=4)
    U.gate(U.gpu_gemv(pl, U.x_dev(L))[None, :], y_ref[:1], f"small outputs, rms {rms:.1e}")
    U.gate(U.gpu_gemm(pl, U.x_dev(L)), y_ref, f"small outputs skinny, rms {rms:.1e}")


@pytest.mark.parametrize("batch", [2, 4, 8, 16])
def test_skinny_batches(batch):
    _run_case(160, 1536, 3, 128, True, batch=batch, seed=batch)
    _run_case(96, 1024, 2, 128, False, batch=batch, seed=batch + 50)


def test_skinny_strided_rows():
    L = bcq_synth.make_layer(128, 1024, 3, group=128, offset=True, batch=3, seed=77)
    pl = U.upload_and_pack(L, max_batch=3)
    Xbig = torch.zeros((3, L.N + 64), dtype=torch.float16, device="cuda")
    Xbig[:, : L.N] = U.x_dev(L)
    Ybig = torch.full((3, L.M + 7), 123.0, dtype=torch.float16, device="cuda")
    bcq.gemm_skinny(pl.desc, pl.packed, Xbig, Xbig.stride(0), Ybig, Ybig.stride(0), 3, pl.workspace)
    torch.cuda.synchronize()
    Y = Ybig.cpu().numpy()
    U.gate(Y[:, : L.M], ref.gemm(L.planes, L.alpha, L.offset, L.x))
    assert np.all(Y[:, L.M:] == 123.0), "columns beyond M must not be written"


def test_outlier_channels():
    """configs[3] activation recipe: 1% of channels scaled x20."""
    _run_case(512, 9216, 3, 128, False, seed=3, outlier_frac=0.01)


@pytest.mark.parametrize("parts", [1, 2, 3, 7])
def test_skinny_k_split_does_not_change_results(parts):
    """The K split of the skinny kernel only changes how partial sums are grouped; on exact
    inputs every split must give the oracle's result bit for bit."""
    L = bcq_synth.make_exact_layer(200, 3584, 3, group=128, offset=True, batch=5, seed=12)
    pl = U.upload_and_pack(L, max_batch=5)
    try:
        bcq.set_option("skinny_parts", parts)
        Y = U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64)
    finally:
        bcq.set_option("skinny_parts", 0)
    # every partial sum is exact in fp32 and in the fixed-point accumulator, so the only
    # rounding is the final one to binary16 (round to nearest even, as numpy does)
    y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    assert np.abs(y_ref).max() < 2 ** 14
    assert np.array_equal(Y, y_ref.astype(np.float16).astype(np.float64))
    assert not pl.workspace.cpu().numpy().any()


def test_skinny_negative_alpha_and_ragged():
    """alpha of either sign (the sign is folded into the plane bits), M % 32 != 0, N % 512 != 0."""
    L = bcq_synth.make_layer(77, 1120, 3, group=1120, offset=True, batch=3, seed=8)
    a = L.alpha.copy()
    a[::2, :, 1] = -a[::2, :, 1]
    a[1::3, :, 0] = -a[1::3, :, 0]
    L.alpha = a
    pl = U.upload_and_pack(L, max_batch=3)
    U.gate(U.gpu_gemm(pl, U.x_dev(L)), ref.gemm(L.planes, L.alpha, L.offset, L.x))
    # the batch-1 kernel on the same layer
    y1 = U.gpu_gemv(pl, U.x_dev(L))
    U.gate(y1[None, :], ref.gemm(L.planes, L.alpha, L.offset, L.x[:1]))


@pytest.mark.parametrize("group", [32, 64])
@pytest.mark.parametrize("q,offset", [(3, False), (2, True), (4, True), (1, False)])
def test_small_groups(group, q, offset):
    """Groups of 32 and 64 columns: 4 or 2 scale sets per 128-column block, batch 1 and skinny."""
    _run_case(203, 1600, q, group, offset, seed=group + q)          # ragged rows and columns
    _run_case(96, 2048, q, group, offset, batch=5, seed=group + q + 1)


@pytest.mark.parametrize("group", [32, 64])
def test_small_groups_exact_and_roundtrip(group):
    """Bit-exact result on exactly representable inputs and pack -> unpack identity for the
    permuted byte order used when a block holds several scaling groups."""
    L = bcq_synth.make_exact_layer(150, 1536, 3, group=group, offset=True, batch=3, seed=group)
    pl = U.upload_and_pack(L, max_batch=3)
    y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    expect = y_ref.astype(np.float16).astype(np.float64)
    xd = U.x_dev(L)
    assert np.array_equal(U.gpu_gemv(pl, xd[0]).astype(np.float64), expect[0])
    assert np.array_equal(U.gpu_gemm(pl, xd).astype(np.float64), expect)
    G = L.N // group
    codes = torch.empty((L.M, L.N), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((L.M, G, L.q), dtype=torch.float16, device="cuda")
    off = torch.empty((L.M, G), dtype=torch.float16, device="cuda")
    bcq.unpack(pl.desc, pl.packed, codes, alpha, off)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), L.codes())
    assert np.array_equal(alpha.cpu().numpy().view(np.uint16), L.alpha.view(np.uint16))
    assert np.array_equal(off.cpu().numpy().view(np.uint16), L.offset.view(np.uint16))


def _rows_of(L, lo, hi):
    codes = U.to_dev(L.codes()[lo:hi])
    alpha = U.to_dev(L.alpha[lo:hi].view(np.uint16).astype(np.int16)).view(torch.float16)
    off = None if L.offset is None else U.to_dev(L.offset[lo:hi].view(np.uint16).astype(np.int16)).view(torch.float16)
    return codes, alpha, off


@pytest.mark.parametrize("group,offset", [(128, True), (64, False)])
def test_pack_rows_builds_the_same_blob_as_one_pack(group, offset):
    """Layers sharing their input, packed range by range into one blob (ranges that do not
    fall on tile boundaries, packed out of order), give byte for byte the blob of a single
    bcq_pack of the stacked layer, hence the same product."""
    L = bcq_synth.make_layer(203, 1152, 3, group=group, offset=offset, seed=41)
    whole = U.upload_and_pack(L)
    fused = bcq.PackedLayer(L.M, L.N, L.q, L.group, L.offset is not None)
    fused.packed.fill_(0xA5)
    for lo, hi in ((150, 203), (0, 37), (37, 150)):
        fused.pack_rows_from(lo, *_rows_of(L, lo, hi))
    torch.cuda.synchronize()
    assert torch.equal(fused.packed, whole.packed)
    y = U.gpu_gemv(fused, U.x_dev(L))
    U.gate(y[None, :], ref.gemm(L.planes, L.alpha, L.offset, L.x), "fused rows")


@pytest.mark.parametrize("option,value", [("skinny_version", 1), ("skinny_version", 2), ("skinny_lds_steps", 3)])
@pytest.mark.parametrize("q,offset", [(3, False), (2, True), (4, True)])
def test_skinny_kernel_variants(option, value, q, offset):
    """Both skinny kernels (alpha folded into the matrix-core operand / +-1 operands from the LDS
    table with alpha applied to the accumulators) and the table/register split of the second,
    on ragged shapes, a multi-part K split and an odd batch."""
    try:
        bcq.set_option(option, value)
        _run_case(203, 3200, q, 128, offset, batch=7, seed=q + value)
        _run_case(64, 1024, q, 256, offset, batch=16, seed=q + value + 1)
        L = bcq_synth.make_exact_layer(96, 2048, q, group=128, offset=offset, batch=3, seed=50 + q)
        pl = U.upload_and_pack(L, max_batch=3)
        expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
        assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), expect)
    finally:
        bcq.set_option(option, 0)


@pytest.mark.parametrize("workgroups", [0, 1, 3, 10, 23])
@pytest.mark.parametrize("q,offset", [(3, True), (1, False), (4, True), (2, False)])
def test_skinny_eight_waves_per_workgroup(workgroups, q, offset):
    """The table kernel with eight waves (eight row tiles) per workgroup, which large layers use: forced
    here on small ragged shapes (10 row tiles = 2 tile groups, the second mostly empty; 3 row tiles;
    M % 32 != 0), any work split, bit-exact on exact inputs, workspace left zero."""
    try:
        bcq.set_option("waves", 8)
        bcq.set_option("workgroups", workgroups)
        L = bcq_synth.make_exact_layer(300, 5120, q, group=128, offset=offset, batch=6, seed=31 + q)
        pl = U.upload_and_pack(L, max_batch=6)
        expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
        assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), expect)
        assert not pl.workspace.cpu().numpy().any()
        _run_case(203, 3200, q, 128, offset, batch=13, seed=q + workgroups)
        _run_case(70, 1536, q, 256, offset, batch=2, seed=q + workgroups + 1)
        _run_case(203, 3200, q, 128, offset, batch=29, seed=q + workgroups + 2)   # 32 columns per pass, eight waves
    finally:
        bcq.set_option("workgroups", 0)
        bcq.set_option("waves", 0)


@pytest.mark.parametrize("workgroups", [0, 3, 10])
@pytest.mark.parametrize("q,offset", [(3, False), (2, True), (1, True), (2, False), (3, True), (4, False)])
def test_skinny_table_kernel_two_column_groups_eight_waves(workgroups, q, offset):
    """17..32 columns on large layers: the table kernel with two groups of 16 columns and eight waves per
    workgroup (16 table copies, one X buffer of two groups; up to three planes, four planes take the four-wave
    kernel).  Forced here on small ragged shapes: bit-exact on exact inputs for any work split, workspace left
    zero, gated on random inputs with ragged batch and rows."""
    try:
        bcq.set_option("waves", 8)
        bcq.set_option("workgroups", workgroups)
        for batch in (17, 32):
            L = bcq_synth.make_exact_layer(300, 5120, q, group=128, offset=offset, batch=batch, seed=61 + q + batch)
            pl = U.upload_and_pack(L, max_batch=batch)
            expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
            assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), expect)
            assert not pl.workspace.cpu().numpy().any()
        _run_case(203, 3200, q, 128, offset, batch=27, seed=q + workgroups + 5)
        _run_case(70, 1536, q, 256, offset, batch=18, seed=q + workgroups + 6)
    finally:
        bcq.set_option("workgroups", 0)
        bcq.set_option("waves", 0)


@pytest.mark.parametrize("workgroups", [0, 1, 3, 7])
@pytest.mark.parametrize("batch", [2, 3, 4])
def test_table_kernel_for_up_to_four_vectors(workgroups, batch):
    """2..4 activation vectors on large layers: sign-sum tables with the four sums side by side, rebuilt along K
    (bcq_lut4.hip).  Forced here on small shapes: ragged rows and columns (a last half slice that is empty or
    partial), fewer tiles than a row group has, one to four planes with and without offset, row-wise scales, any
    work split; bit for bit the oracle's result (one binary16 rounding) on exact inputs, workspace left zero;
    gate on random inputs with outlier channels; padded rows of X and Y."""
    try:
        bcq.set_option("skinny_version", 3)
        bcq.set_option("workgroups", workgroups)
        for (M, N, q, off, group) in [(96, 2048, 3, False, 128), (300, 5120, 3, True, 128), (70, 1536, 2, True, 128),
                                      (1000, 2560, 1, False, 128), (203, 3200, 4, False, 128), (96, 2048, 3, True, 2048),
                                      (40, 1024, 2, False, 256), (2100, 1024, 3, False, 128)]:
            L = bcq_synth.make_exact_layer(M, N, q, group=group, offset=off, batch=batch, seed=M + q + batch)
            pl = U.upload_and_pack(L, max_batch=batch)
            expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
            assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), expect), (M, N, q, off, group)
            assert not pl.workspace.cpu().numpy().any()
        _run_case(600, 4608, 3, 128, True, batch=batch, seed=batch + workgroups, outlier_frac=0.01)
        L = bcq_synth.make_exact_layer(150, 3072, 3, group=128, offset=True, batch=batch, seed=77)
        pl = U.upload_and_pack(L, max_batch=batch)
        expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
        X = torch.zeros((batch, L.N + 64), dtype=torch.float16, device="cuda")
        X[:, :L.N] = U.x_dev(L)
        Y = torch.full((batch, L.M + 10), 3.0, dtype=torch.float16, device="cuda")
        bcq.gemm_skinny(pl.desc, pl.packed, X, X.stride(0), Y, Y.stride(0), batch, pl.workspace)
        torch.cuda.synchronize()
        assert np.array_equal(Y[:, :L.M].cpu().numpy().astype(np.float64), expect)
        assert torch.all(Y[:, L.M:] == 3.0)
    finally:
        bcq.set_option("workgroups", 0)
        bcq.set_option("skinny_version", 0)


@pytest.mark.parametrize("workgroups", [0, 1, 3, 7, 50])
def test_two_vector_table_kernel(workgroups):
    """Two activation vectors on layers from 2048 tiles on: the GEMV's decomposition with both vectors' sign sums
    in one table entry (bcq_gemv2.hip).  Forced here on small shapes: ragged rows and columns, a single column
    slice (no split-K), fewer tiles than waves, one to four planes with and without offset, row-wise scales and
    groups of 256, any grid size; bit for bit the oracle's result (one binary16 rounding) on exact inputs, twice in
    a row, workspace left zero; gate on random inputs with outlier channels; padded rows of X and Y; binary16
    subnormal scales."""
    try:
        bcq.set_option("skinny_version", 5)
        bcq.set_option("workgroups", workgroups)
        for (M, N, q, off, group) in [(96, 2048, 3, False, 128), (300, 5120, 3, True, 128), (70, 1536, 2, True, 128),
                                      (1000, 2560, 1, False, 128), (203, 3200, 4, True, 128), (96, 2048, 3, True, 2048),
                                      (40, 1024, 3, False, 128), (520, 512, 2, True, 128), (777, 6656, 3, False, 256),
                                      (33, 640, 4, False, 128)]:
            L = bcq_synth.make_exact_layer(M, N, q, group=group, offset=off, batch=2, seed=M + q)
            pl = U.upload_and_pack(L, max_batch=2)
            expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
            for _ in range(2):
                assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), expect), (M, N, q, off, group)
            assert pl.workspace is None or not pl.workspace.cpu().numpy().any()
        _run_case(600, 4608, 3, 128, True, batch=2, seed=workgroups, outlier_frac=0.01)
        _run_case(1024, 4096, 2, 128, False, batch=2, seed=workgroups + 1)
        L = bcq_synth.make_exact_layer(150, 3072, 3, group=128, offset=True, batch=2, seed=77)
        pl = U.upload_and_pack(L, max_batch=2)
        expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
        X = torch.zeros((2, L.N + 64), dtype=torch.float16, device="cuda")
        X[:, :L.N] = U.x_dev(L)
        Y = torch.full((2, L.M + 10), 3.0, dtype=torch.float16, device="cuda")
        bcq.gemm_skinny(pl.desc, pl.packed, X, X.stride(0), Y, Y.stride(0), 2, pl.workspace)
        torch.cuda.synchronize()
        assert np.array_equal(Y[:, :L.M].cpu().numpy().astype(np.float64), expect)
        assert torch.all(Y[:, L.M:] == 3.0)
        # every alpha and offset a binary16 subnormal: exact in binary32, so bit for bit the oracle's rounded result
        L = bcq_synth.make_exact_layer(150, 2048, 3, group=128, offset=True, batch=2, seed=92)
        rng = np.random.default_rng(7)
        L.alpha = rng.integers(1, 1024, size=L.alpha.shape, dtype=np.uint16).view(np.float16)
        z = rng.integers(1, 1024, size=L.offset.shape, dtype=np.uint16) | (rng.integers(0, 2, size=L.offset.shape, dtype=np.uint16) << 15)
        L.offset = z.view(np.float16)
        y_ref = ref.gemm(L.planes, L.alpha, L.offset, L.x)
        assert np.abs(y_ref).max() > 2.0 ** -12, "the scales must matter"
        pl = U.upload_and_pack(L, max_batch=2)
        assert np.array_equal(U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64), y_ref.astype(np.float16).astype(np.float64))
    finally:
        bcq.set_option("workgroups", 0)
        bcq.set_option("skinny_version", 0)


@pytest.mark.parametrize("workgroups", [1, 4, 7, 11, 29])
@pytest.mark.parametrize("version", [1, 2])
def test_skinny_work_split_does_not_change_results(workgroups, version):
    """The skinny kernel cuts its (tile group, column slice) units into equal contiguous ranges, one
    per workgroup; a range may end inside a tile group and continue in the next.  Any number of
    workgroups gives the same bits on exact inputs (10 row tiles = 3 tile groups, the last one
    partly empty; 10 column slices)."""
    L = bcq_synth.make_exact_layer(300, 5120, 3, group=128, offset=True, batch=6, seed=31)
    pl = U.upload_and_pack(L, max_batch=6)
    expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
    try:
        bcq.set_option("skinny_version", version)
        bcq.set_option("workgroups", workgroups)
        Y = U.gpu_gemm(pl, U.x_dev(L)).astype(np.float64)
    finally:
        bcq.set_option("workgroups", 0)
        bcq.set_option("skinny_version", 0)
    assert np.array_equal(Y, expect)
    assert not pl.workspace.cpu().numpy().any()


def test_graph_replay_matches_eager():
    """The entry points only enqueue kernels (the workspace fill is a kernel, not a memset node), so
    a captured sequence -- workspace init, GEMV, skinny GEMM -- can be replayed: every replay, with
    eager calls and synchronisations in between, reproduces the eager results bit for bit."""
    L = bcq_synth.make_layer(260, 2560, 3, group=128, offset=True, batch=5, seed=61)
    pl = U.upload_and_pack(L, max_batch=5)
    X = U.x_dev(L)
    y_eager = pl.gemv(X[0]).clone()
    Y_eager = pl.gemm_skinny(X).clone()
    torch.cuda.synchronize()
    y_g = torch.zeros_like(y_eager)
    Y_g = torch.zeros_like(Y_eager)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            bcq.workspace_init(pl.workspace)
            pl.gemv(X[0], y_g)
            pl.gemm_skinny(X, Y_g)
    for rep in range(4):
        y_g.fill_(7.0)
        Y_g.fill_(7.0)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            g.replay()
        stream.synchronize()
        assert torch.equal(y_g, y_eager), rep
        assert torch.equal(Y_g, Y_eager), rep
        # eager work of the program between replays
        assert torch.equal(pl.gemm_skinny(X), Y_eager)
        torch.cuda.synchronize()


@pytest.mark.parametrize("version", [0, 2])
@pytest.mark.parametrize("batch", [17, 24, 32, 33, 50, 64])
@pytest.mark.parametrize("q,offset,group", [(3, False, 128), (2, True, 128), (4, True, 256), (3, True, 64)])
def test_wide_batches(batch, q, offset, group, version):
    """17..64 activation vectors: the expanded operands are shared between groups of 16 columns, up to 64
    per pass (default: the kernel that folds alpha into A; version 2: the table kernel, q = 4: 32 per
    pass); groups of 64 columns take one pass per 16."""
    try:
        bcq.set_option("skinny_version", version)
        _run_case(203, 2560, q, group, offset, batch=batch, seed=batch + q)
    finally:
        bcq.set_option("skinny_version", 0)


def test_wide_batch_exact_and_strided():
    L = bcq_synth.make_exact_layer(150, 3072, 3, group=128, offset=True, batch=40, seed=77)
    pl = U.upload_and_pack(L, max_batch=40)
    expect = ref.gemm(L.planes, L.alpha, L.offset, L.x).astype(np.float16).astype(np.float64)
    X = torch.zeros((40, L.N + 64), dtype=torch.float16, device="cuda")
    X[:, :L.N] = U.x_dev(L)
    Y = torch.full((40, L.M + 10), 3.0, dtype=torch.float16, device="cuda")
    bcq.gemm_skinny(pl.desc, pl.packed, X, X.stride(0), Y, Y.stride(0), 40, pl.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(Y[:, :L.M].cpu().numpy().astype(np.float64), expect)
    assert torch.all(Y[:, L.M:] == 3.0)
    assert not pl.workspace.cpu().numpy().any()


def test_maximum_column_count():
    """N = 523776 = 1023 column slices, the most the 10-bit arrival count of the split-K word holds
    (one more slice is refused by the descriptor check): GEMV and skinny kernel."""
    N = 1023 * 512
    d = bcq.Desc(40, N + 512, 2, 128, 0, 0)
    assert bcq.packed_bytes(d) == 0
    _run_case(40, N, 2, 128, True, seed=3)
    _run_case(40, N, 2, 128, True, batch=3, seed=4)


@pytest.mark.parametrize("q,offset", [(3, True), (2, False), (4, True)])
def test_row_wise_parameters(q, offset):
    """group = N, the paper's setting (quantisation parameters fixed per row): scale records are
    stored once per row; GEMV, both skinny kernels, wide batch, pack/unpack round trip, fused rows."""
    for M, N in ((203, 2560), (64, 96), (100, 7168)):
        _run_case(M, N, q, N, offset, seed=M + q)
        _run_case(M, N, q, N, offset, batch=5, seed=M + q + 1)
    _run_case(150, 3072, q, 3072, offset, batch=40, seed=q)
    try:
        bcq.set_option("skinny_version", 1)
        _run_case(150, 3072, q, 3072, offset, batch=9, seed=q + 9)
    finally:
        bcq.set_option("skinny_version", 0)
    L = bcq_synth.make_layer(77, 1120, q, group=1120, offset=offset, seed=8 + q)
    pl = U.upload_and_pack(L)
    codes = torch.empty((L.M, L.N), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((L.M, 1, L.q), dtype=torch.float16, device="cuda")
    off = torch.empty((L.M, 1), dtype=torch.float16, device="cuda") if offset else None
    bcq.unpack(pl.desc, pl.packed, codes, alpha, off)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), L.codes())
    assert np.array_equal(alpha.cpu().numpy().view(np.uint16), L.alpha.view(np.uint16))
    if offset:
        assert np.array_equal(off.cpu().numpy().view(np.uint16), L.offset.view(np.uint16))
    fused = bcq.PackedLayer(L.M, L.N, L.q, L.group, offset)
    fused.packed.fill_(0x5A)
    for lo, hi in ((30, 77), (0, 30)):
        fused.pack_rows_from(lo, *_rows_of(L, lo, hi))
    torch.cuda.synchronize()
    assert torch.equal(fused.packed, pl.packed)
