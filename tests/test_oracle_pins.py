"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign, wrong bit order,
wrong group index, transposed operand) fails at least one of them.
"""
import os

import numpy as np
import pytest

import bcq_synth
from oracle import fuse, ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key.strip()] = [float(v) for v in vals.split()]
    return out


# --------------------------------------------------------------------------
# binary16 widening against numpy (library routine, all bit patterns)
# --------------------------------------------------------------------------
def test_half_to_double_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = ref.half_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# --------------------------------------------------------------------------
# paper values: Eq. 6, 8, 9, 10, 11
# --------------------------------------------------------------------------
def test_eq6_worked_example():
    g = read_golden("eq6_nearest_bcchoice.txt")
    got = fuse.nearest_bcchoice(np.array(g["W_int"], dtype=np.int64), [int(v) for v in g["BCchoice"]])
    assert got.tolist() == [int(v) for v in g["W_q"]]


def test_eq9_three_bit_identity():
    g = read_golden("eq8_to_eq11_constants.txt")
    alphas, centre = fuse.linear_plane_alphas(3)
    assert alphas.tolist() == g["eq9_alpha"]
    assert centre == g["eq9_centre"][0]
    W_int = np.array(g["eq9_W_int"], dtype=np.int64)
    signs = fuse.int_to_signs(W_int, 3)                      # [3][8]
    assert np.array_equal((alphas[:, None] * signs).sum(0) + centre, W_int)
    # each integer has its own sign triple
    assert len({tuple(signs[:, t]) for t in range(8)}) == 8


def test_eq10_tied_planes_set():
    g = read_golden("eq8_to_eq11_constants.txt")
    part = ((1,), (2, 3))
    assert part in fuse.all_partitions(3, 2)
    assert fuse.fused_alphas(part).tolist() == g["eq10_alpha_hat"]
    assert fuse.bcchoice(part, 3) == [int(v) for v in g["eq10_representable"]]
    # same set as the BCchoice of the Eq. 6 example
    assert fuse.bcchoice(part, 3) == [int(v) for v in read_golden("eq6_nearest_bcchoice.txt")["BCchoice"]]


def test_partition_count_is_stirling():
    # S(5,3) = 25, S(3,2) = 3, S(4,2) = 7
    assert len(fuse.all_partitions(5, 3)) == 25
    assert len(fuse.all_partitions(3, 2)) == 3
    assert len(fuse.all_partitions(4, 2)) == 7


def test_eq8_two_bit_linear_grid():
    """Eq. 8: alpha = {S, S/2} spans the 2-bit signed grid; the sum of +-alpha
    equals (W_int + 1/2) S, i.e. the grid up to the half-step the offset holds."""
    g = read_golden("eq8_to_eq11_constants.txt")
    S = 0.375
    a = np.array(g["eq8_alpha_over_S"]) * S
    vals = sorted(s1 * a[0] + s2 * a[1] for s1 in (-1, 1) for s2 in (-1, 1))
    assert vals == [(w + 0.5) * S for w in g["eq8_W_int"]]
    # through the oracle: planes of (W_int + 2) in {0..3}, n = 2 linear planes
    W_int = np.tile(np.array(g["eq8_W_int"], dtype=np.int64), 8)[None, :]   # [1][32]
    part = ((1,), (2,))
    planes, alpha, z = fuse.fuse(W_int + 2, np.full((1, 1), S), np.full((1, 1), -2 * S), part, 2, 32)
    assert np.array_equal(np.sort(alpha[0, 0])[::-1], a)
    W = ref.dequant(planes, alpha.astype(np.float16), z.astype(np.float16))
    assert np.array_equal(W, S * W_int)


@pytest.mark.parametrize("n,q", [(3, 2), (3, 3), (4, 2), (5, 3), (5, 2), (4, 4)])
def test_round_trip_fused_form_is_exact(n, q):
    """Eq. 9-11 round trip: nearest-BCchoice integers, fused to q planes and
    dequantised by the oracle, equal S * W_q + qbias exactly (S a power of two
    and qbias a multiple of S/2 keep every operand exact in fp16)."""
    rng = np.random.default_rng(100 * n + q)
    M, N, group = 12, 256, 64
    G = N // group
    for part in fuse.all_partitions(n, q)[:6]:
        S = 2.0 ** rng.integers(-8, -3, size=(M, G))
        qbias = rng.integers(-40, 40, size=(M, G)) * S / 2
        W_int = rng.integers(0, 2 ** n, size=(M, N))
        choice = fuse.bcchoice(part, n)
        assert len(choice) == 2 ** q
        W_q = fuse.nearest_bcchoice(W_int, choice)
        assert set(np.unique(W_q)) <= set(choice)
        assert np.all(np.abs(W_q - W_int) <= np.abs(W_int[..., None] - np.array(choice)).min(-1))
        planes, alpha, z = fuse.fuse(W_q, S, qbias, part, n, group)
        a16, z16 = alpha.astype(np.float16), z.astype(np.float16)
        assert np.array_equal(a16.astype(np.float64), alpha)
        assert np.array_equal(z16.astype(np.float64), z)
        W = ref.dequant(planes, a16, z16)
        want = np.repeat(S, group, axis=1) * W_q + np.repeat(qbias, group, axis=1)
        assert np.array_equal(W, want)


def test_round_trip_general_scale_within_half_ulp_of_offset():
    """Same round trip with an arbitrary fp16 S: alpha_hat = S*integer/2 stays
    exact when S has few mantissa bits; z is rounded to fp16, so the result is
    within half an fp16 ulp of z of the linear reconstruction."""
    rng = np.random.default_rng(7)
    n, q, M, N, group = 3, 2, 8, 128, 128
    part = ((1,), (2, 3))
    S = (rng.integers(16, 32, size=(M, 1)) / 1024.0)          # 5 significant bits
    qbias = rng.normal(0, 0.05, size=(M, 1)).astype(np.float16).astype(np.float64)
    W_q = fuse.nearest_bcchoice(rng.integers(0, 8, size=(M, N)), fuse.bcchoice(part, n))
    planes, alpha, z = fuse.fuse(W_q, S, qbias, part, n, group)
    a16 = alpha.astype(np.float16)
    assert np.array_equal(a16.astype(np.float64), alpha)
    z16 = z.astype(np.float16)
    W = ref.dequant(planes, a16, z16)
    want = S * W_q + qbias
    ulp = np.spacing(np.abs(z16)).astype(np.float64)
    assert np.all(np.abs(W - want) <= 0.5 * ulp + 1e-300)
    # Eq. 11 constants
    g = read_golden("eq8_to_eq11_constants.txt")
    assert np.allclose(np.sort(alpha[:, 0, :] / S, axis=1), np.sort(g["eq11_alpha_hat_over_S"]))
    assert np.array_equal(z, g["eq11_offset_centre"][0] * S + qbias)


# --------------------------------------------------------------------------
# special cases that reduce to textbook routines
# --------------------------------------------------------------------------
def test_q1_sign_matrix_against_int64_matvec():
    rng = np.random.default_rng(1)
    M, N = 48, 320
    planes = rng.integers(0, 2 ** 32, size=(1, M, N // 32), dtype=np.uint32)
    alpha = np.ones((M, 1, 1), dtype=np.float16)
    x = rng.integers(-9, 10, size=(3, N)).astype(np.float16)
    Y = ref.gemm(planes, alpha, None, x)
    bits = np.unpackbits(planes[0].view(np.uint8), axis=1, bitorder="little").astype(np.int64)
    sign = 2 * bits - 1
    want = x.astype(np.int64) @ sign.T                        # [3][M]
    assert np.array_equal(Y, want.astype(np.float64))


def test_popcount_closed_form_with_all_ones_input():
    L = bcq_synth.make_layer(40, 384, 3, group=128, offset=True, seed=3)
    x = np.ones((1, L.N), dtype=np.float16)
    Y = ref.gemm(L.planes, L.alpha, L.offset, x)[0]
    a = L.alpha.astype(np.float64)
    z = L.offset.astype(np.float64)
    G = L.N // L.group
    want = np.zeros(L.M)
    for m in range(L.M):
        for grp in range(G):
            for i in range(L.q):
                words = L.planes[i, m, grp * 4:(grp + 1) * 4]
                pc = sum(bin(int(w)).count("1") for w in words)
                want[m] += a[m, grp, i] * (2 * pc - L.group)
            want[m] += L.group * z[m, grp]
    assert np.allclose(Y, want, rtol=1e-13, atol=1e-15)


def test_column_probe_fixes_bit_order_and_group_index():
    """x = e_k returns column k of W: +-alpha summed, plus z.  A planted single
    bit pins LSB-first order inside a word and the word/group index."""
    M, N, q, group = 4, 256, 2, 64
    planes = np.zeros((q, M, N // 32), dtype=np.uint32)
    k_hot, m_hot = 32 * 5 + 3, 2                              # word 5, bit 3 -> column 163, group 2
    planes[1, m_hot, 5] = np.uint32(1 << 3)
    alpha = np.zeros((M, N // group, q), dtype=np.float16)
    alpha[:, :, 0] = np.arange(1, 5)[None, :]                 # plane 0 scale = group index + 1
    alpha[:, :, 1] = 0.25
    # offset = 16 m + 3 grp: its group term must not cancel the plane-0 scale's (a mutation check found that
    # 8 m + grp did, which left a shifted group index unnoticed by this pin)
    z = (np.arange(M)[:, None] * 16 + 3 * np.arange(N // group)[None, :]).astype(np.float16)
    for k in (0, 31, 63, 64, k_hot, k_hot + 1, 255):
        x = np.zeros((1, N), dtype=np.float16)
        x[0, k] = 1.0
        y = ref.gemm(planes, alpha, z, x)[0]
        for m in range(M):
            grp = k // group
            s1 = 1.0 if (m == m_hot and k == k_hot) else -1.0
            want = -(grp + 1) + 0.25 * s1 + (16 * m + 3 * grp)
            assert y[m] == want, (k, m)


def test_transposition_would_be_caught():
    """Y is [b][M] with Y[j][m] = W[m,:] . X[j,:] -- checked against numpy's
    matmul on the dequantised matrix (library routine as the step)."""
    L = bcq_synth.make_layer(24, 160 * 2, 3, group=32, offset=True, batch=5, seed=11)
    W = ref.dequant(L.planes, L.alpha, L.offset)
    want = L.x.astype(np.float64) @ W.T
    got = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    assert got.shape == (5, 24)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(ref.dense_matmul(W, L.x), want, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------
# brute force
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,N", [(32, 32), (33, 96), (64, 256), (17, 128)])
@pytest.mark.parametrize("q", [1, 2, 3])
def test_gemm_against_brute_force(M, N, q):
    for group in sorted({32, 64, 128, N}):
        if N % group:
            continue
        for offset in (False, True):
            L = bcq_synth.make_layer(M, N, q, group=group, offset=offset, batch=2, seed=M + N + q)
            a = ref.gemm(L.planes, L.alpha, L.offset, L.x)
            b = ref.brute(L.planes, L.alpha, L.offset, L.x)
            scale = np.abs(a).max()
            assert np.max(np.abs(a - b)) <= 1e-12 * scale


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
def _layer(seed=5, **kw):
    return bcq_synth.make_layer(32, 256, 3, group=64, offset=True, batch=2, seed=seed, **kw)


def test_linearity_in_x():
    L = _layer()
    x2 = bcq_synth.make_layer(32, 256, 3, group=64, batch=2, seed=99).x
    # fp16 sums may round; build the combination from exactly representable halves
    xa = (L.x.astype(np.float64) / 4).astype(np.float16)
    xb = (x2.astype(np.float64) / 4).astype(np.float16)
    ya = ref.gemm(L.planes, L.alpha, L.offset, xa)
    yb = ref.gemm(L.planes, L.alpha, L.offset, xb)
    W = ref.dequant(L.planes, L.alpha, L.offset)
    yab = (xa.astype(np.float64) + xb.astype(np.float64)) @ W.T
    assert np.allclose(ya + yb, yab, rtol=1e-12, atol=1e-12)


def test_flipping_a_plane_negates_its_alpha():
    L = _layer()
    y0 = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    planes = L.planes.copy()
    planes[1] = ~planes[1]
    alpha = L.alpha.copy()
    alpha[:, :, 1] = -alpha[:, :, 1]
    assert np.array_equal(ref.dequant(planes, alpha, L.offset), ref.dequant(L.planes, L.alpha, L.offset))
    assert np.array_equal(ref.gemm(planes, alpha, L.offset, L.x), y0)


def test_plane_permutation_and_zero_alpha_plane():
    L = _layer()
    y0 = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    perm = [2, 0, 1]
    y1 = ref.gemm(L.planes[perm], L.alpha[:, :, perm], L.offset, L.x)
    assert np.allclose(y0, y1, rtol=1e-13, atol=1e-14)
    alpha = L.alpha.copy()
    alpha[:, :, 2] = 0
    y3 = ref.gemm(L.planes, alpha, L.offset, L.x)
    y2 = ref.gemm(L.planes[:2], np.ascontiguousarray(alpha[:, :, :2]), L.offset, L.x)
    assert np.array_equal(y3, y2)


def test_doubling_alpha_doubles_the_plane_part_and_rows_commute():
    L = _layer()
    y_off = ref.gemm(L.planes, np.zeros_like(L.alpha), L.offset, L.x)
    y1 = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    a2 = (L.alpha.astype(np.float64) * 2).astype(np.float16)
    y2 = ref.gemm(L.planes, a2, L.offset, L.x)
    assert np.allclose(y2 - y_off, 2 * (y1 - y_off), rtol=1e-12, atol=1e-13)
    rp = np.random.default_rng(0).permutation(L.M)
    yp = ref.gemm(L.planes[:, rp], L.alpha[rp], L.offset[rp], L.x)
    assert np.array_equal(yp, y1[:, rp])


def test_no_offset_equals_zero_offset():
    L = _layer()
    assert np.array_equal(ref.gemm(L.planes, L.alpha, None, L.x),
                          ref.gemm(L.planes, L.alpha, np.zeros_like(L.offset), L.x))


def test_subnormal_alpha_is_kept():
    M, N = 2, 32
    planes = np.full((1, M, 1), 0xFFFFFFFF, dtype=np.uint32)
    alpha = np.array([1, 0x03FF], dtype=np.uint16).view(np.float16).reshape(M, 1, 1)
    x = np.ones((1, N), dtype=np.float16)
    y = ref.gemm(planes, alpha, None, x)[0]
    assert y[0] == 32 * 2.0 ** -24 and y[1] == 32 * 1023 * 2.0 ** -24


def test_exact_layer_is_integer_valued_and_matches_brute():
    L = bcq_synth.make_exact_layer(32, 512, 3, group=128, offset=True, batch=2, seed=4)
    a = ref.gemm(L.planes, L.alpha, L.offset, L.x)
    b = ref.brute(L.planes, L.alpha, L.offset, L.x)
    assert np.array_equal(a, b)
    assert np.array_equal(a * 4, np.round(a * 4))


def test_synth_codes_round_trip():
    L = bcq_synth.make_layer(16, 96, 3, group=32, seed=2)
    codes = L.codes()
    assert codes.max() < 8
    assert np.array_equal(bcq_synth.codes_to_planes(codes, 3), L.planes)
    assert codes[3, 37] == sum(((int(L.planes[i, 3, 1]) >> 5) & 1) << i for i in range(3))
