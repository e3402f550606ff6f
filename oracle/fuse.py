"""Oracle for the step that feeds the hot path: turning the two-step
quantisation result into one binary coding (paper Sec. II-B Eq. 6 and
Sec. II-D Eq. 8-11).  TEST INFRASTRUCTURE; fp64 / exact integers, pure numpy.

Notation follows the paper: n = bits of the intermediate linear quantisation,
q = number of binary-coding planes, S = linear scale, qbias = linear bias,
W_int in {0 .. 2^n - 1}.

Readings where the paper is silent (listed in the design notes as well):
  * a stored bit 1 means b = +1, bit 0 means b = -1;
  * the tied-plane sets are the partitions of the n linear planes into q
    non-empty classes; Eq. 10 is the partition {1},{2,3};
  * nearest-BCchoice ties go to the smaller integer (the paper's example has
    no tie);
  * in the output, plane 0 carries the largest fused alpha.
"""
import itertools

import numpy as np


def linear_plane_alphas(n):
    """Eq. 9: W_int = sum_{i=1..n} alpha_i b_i + (2^n - 1)/2, alpha_i = 2^(i-2).

    Returns (alphas[n] with alphas[i-1] = 2^(i-2), centre (2^n - 1)/2)."""
    return np.array([2.0 ** (i - 2) for i in range(1, n + 1)]), (2 ** n - 1) / 2.0


def int_to_signs(W_int, n):
    """Eq. 9: b_i = +1 where bit (i-1) of W_int is set, else -1; shape [n, ...]."""
    W_int = np.asarray(W_int, dtype=np.int64)
    return np.stack([2 * ((W_int >> (i - 1)) & 1) - 1 for i in range(1, n + 1)])


def all_partitions(n, q):
    """All ways to tie the n linear planes (numbered 1..n) into q non-empty
    classes (Eq. 10 is ((1,), (2, 3)) for n = 3, q = 2)."""
    out = set()
    for labels in itertools.product(range(q), repeat=n):
        if len(set(labels)) != q:
            continue
        classes = tuple(sorted(tuple(i + 1 for i in range(n) if labels[i] == c) for c in range(q)))
        out.add(classes)
    return sorted(out)


def fused_alphas(partition):
    """Eq. 10: alpha_hat of a class = sum of 2^(i-2) over the planes tied in it."""
    return np.array([sum(2.0 ** (i - 2) for i in cls) for cls in partition])


def bcchoice(partition, n):
    """The integers representable when the planes of each class share one sign:
    sum_c (+-) alpha_hat_c + (2^n - 1)/2  (Eq. 10)."""
    ah = fused_alphas(partition)
    centre = (2 ** n - 1) / 2.0
    vals = set()
    for signs in itertools.product((-1.0, 1.0), repeat=len(partition)):
        v = float(np.dot(signs, ah)) + centre
        assert v == int(v)
        vals.add(int(v))
    return sorted(vals)


def nearest_bcchoice(W_int, choice):
    """Eq. 6: replace every integer by the nearest member of BCchoice
    (ties to the smaller member)."""
    W_int = np.asarray(W_int, dtype=np.int64)
    choice = np.array(sorted(choice), dtype=np.int64)
    dist = np.abs(W_int[..., None] - choice)          # [..., |choice|]
    return choice[np.argmin(dist, axis=-1)]           # argmin takes the first (smaller) on ties


def linear_quantize(W, S, qbias, n):
    """Step 1 of Eq. 5 read so that it inverts the dequantisation rule
    W_hat = S * W_int + qbias stated with Eq. 8: round-half-even of
    (W - qbias)/S, clamped to 0 .. 2^n - 1."""
    W_int = np.rint((np.asarray(W, dtype=np.float64) - qbias) / S)
    return np.clip(W_int, 0, 2 ** n - 1).astype(np.int64)


def fuse(W_q, S, qbias, partition, n, group):
    """Eq. 11: the fused binary coding of integers W_q (members of the
    partition's BCchoice) under per-group S and qbias.

    W_q [M][N] ints; S, qbias [M][N/group] fp64.
    Returns planes [q][M][N/32] uint32 (LSB first along N), alpha_hat
    [M][G][q] fp64, z [M][G] fp64 with
        alpha_hat_c = S * sum_{i in class c} 2^(i-2),   z = (2^n - 1)/2 * S + qbias,
    classes ordered by descending alpha_hat."""
    W_q = np.asarray(W_q, dtype=np.int64)
    M, N = W_q.shape
    G = N // group
    S = np.asarray(S, dtype=np.float64).reshape(M, G)
    qbias = np.asarray(qbias, dtype=np.float64).reshape(M, G)
    ah = fused_alphas(partition)
    order = np.argsort(-ah, kind="stable")
    signs = int_to_signs(W_q, n)                       # [n][M][N]
    q = len(partition)
    planes = np.zeros((q, M, N // 32), dtype=np.uint32)
    alpha = np.empty((M, G, q), dtype=np.float64)
    for out_idx, c in enumerate(order):
        cls = partition[c]
        s = signs[cls[0] - 1]
        for i in cls[1:]:
            if not np.array_equal(signs[i - 1], s):
                raise ValueError("W_q is not representable with this partition")
        bits = (s > 0).astype(np.uint32).reshape(M, N // 32, 32)
        planes[out_idx] = (bits << np.arange(32, dtype=np.uint32)).sum(axis=2, dtype=np.uint64).astype(np.uint32)
        alpha[:, :, out_idx] = S * ah[c]
    z = (2 ** n - 1) / 2.0 * S + qbias
    return planes, alpha, z
