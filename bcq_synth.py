"""Seeded synthetic inputs shared by the oracle-side tests, the GPU parity
tests and the bench.  Holds no arithmetic of the method: only random draws and
re-encodings of the same bits (plane words <-> per-weight codes).

Canonical layout (what the oracle reads, and what bcq_pack consumes as codes):
    planes [q][M][N/32] uint32, LSB first along N (bit j of word w = column 32w+j)
    codes  [M][N] uint8, bit i of a code = the bit of plane i
    alpha  [M][N/g][q] float16,  offset [M][N/g] float16 or None
    x      [b][N] float16

Recipe (stands in for the OPT / Llama-2 layers the paper measures; only the
layer shapes are taken from those models):
    rng = Generator(PCG64(seed)); draw order planes, alpha, offset, x
    planes: iid uniform bits;  alpha: |N(0, 0.02)| sorted descending over the
    plane axis, cast to fp16;  offset: N(0, 0.01) -> fp16;  x: N(0, 1) -> fp16,
    optionally a fraction of channels (same for every batch row) scaled x20
    before the cast.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class Layer:
    M: int
    N: int
    q: int
    group: int
    planes: np.ndarray            # [q][M][N/32] uint32
    alpha: np.ndarray             # [M][G][q] float16
    offset: Optional[np.ndarray]  # [M][G] float16 or None
    x: np.ndarray                 # [b][N] float16

    @property
    def batch(self):
        return self.x.shape[0]

    def codes(self):
        return planes_to_codes(self.planes)

    def weight_bytes(self):
        G = self.N // self.group
        nbytes = self.q * self.M * self.N // 8 + self.q * self.M * G * 2
        if self.offset is not None:
            nbytes += self.M * G * 2
        return nbytes


def planes_to_codes(planes):
    """[q][M][N/32] uint32 -> [M][N] uint8 with bit i of the code = plane i's bit."""
    q, M, words = planes.shape
    codes = np.zeros((M, words * 32), dtype=np.uint8)
    for i in range(q):
        bits = np.unpackbits(np.ascontiguousarray(planes[i]).view(np.uint8), axis=1, bitorder="little")
        codes |= (bits << i).astype(np.uint8)
    return codes


def codes_to_planes(codes, q):
    """Inverse of planes_to_codes."""
    M, N = codes.shape
    planes = np.empty((q, M, N // 32), dtype=np.uint32)
    for i in range(q):
        bits = ((codes >> i) & 1).astype(np.uint8)
        planes[i] = np.packbits(bits, axis=1, bitorder="little").view(np.uint32)
    return planes


def make_layer(M, N, q, group=128, offset=False, batch=1, seed=0,
               outlier_frac=0.0, outlier_scale=20.0):
    """The benchmark recipe (see module docstring)."""
    assert N % 32 == 0 and N % group == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    G = N // group
    planes = rng.integers(0, 2 ** 32, size=(q, M, N // 32), dtype=np.uint32)
    alpha = np.abs(rng.normal(0.0, 0.02, size=(M, G, q)))
    alpha = -np.sort(-alpha, axis=2)
    alpha = alpha.astype(np.float16)
    off = rng.normal(0.0, 0.01, size=(M, G)).astype(np.float16) if offset else None
    x = rng.normal(0.0, 1.0, size=(batch, N))
    if outlier_frac > 0.0:
        n_out = int(round(outlier_frac * N))
        idx = rng.choice(N, size=n_out, replace=False)
        x[:, idx] *= outlier_scale
    x = x.astype(np.float16)
    return Layer(M, N, q, group, planes, alpha, off, x)


def make_exact_layer(M, N, q, group=128, offset=False, batch=1, seed=0):
    """Inputs on which fp16, fp32 and fp64 arithmetic all give the same,
    exactly representable answer: alpha in {1/4, 1/2, 1, 2}, x small integers,
    offset small integers.  Any difference between two correct evaluations is
    then an indexing bug, not rounding."""
    rng = np.random.Generator(np.random.PCG64(seed))
    G = N // group
    planes = rng.integers(0, 2 ** 32, size=(q, M, N // 32), dtype=np.uint32)
    alpha = (2.0 ** rng.integers(-2, 2, size=(M, G, q))).astype(np.float16)
    off = rng.integers(-2, 3, size=(M, G)).astype(np.float16) if offset else None
    x = rng.integers(-2, 3, size=(batch, N)).astype(np.float16)
    return Layer(M, N, q, group, planes, alpha, off, x)


# Layer shapes (M out x N in) of the models the workloads are shaped after.
OPT_30B = {"attn_proj": (7168, 7168), "fc1": (28672, 7168), "fc2": (7168, 28672)}
OPT_66B = {"attn_proj": (9216, 9216), "fc1": (36864, 9216), "fc2": (9216, 36864)}
LLAMA2_70B_BLOCK = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192),
                    ("o", 8192, 8192), ("gate", 28672, 8192), ("up", 28672, 8192),
                    ("down", 8192, 28672)]
