// Internal geometry of the packed weight blob (layout version 2), shared by the
// pack, GEMV and skinny kernels of this library.  Not part of the public ABI.
//
// The weight of Eq. 11 (q sign planes, per-group alpha, optional offset) is cut
// into tiles of 32 rows x 512 columns.  A tile is what one 64-lane wavefront
// consumes per step of the GEMV:
//
//   lane l = 16*h + r  (h = 0..3, r = 0..15) owns, for both row halves t = 0,1,
//   the 128-column block kb = 4*slice + h of row 32*tile + 16*t + r.
//
//   tile bytes:
//     [t][plane i][lane l]  16 bytes : the 128 sign bits of (row, block kb, plane i)
//                                      byte j holds the 8 columns 128*kb + 8*c + (0..7),
//                                      c = chunk_of_byte(j, r, sub), least-significant bit =
//                                      lowest column.  For sub = 1 this is (j + r) mod 16;
//                                      in every case the 16 lanes of a row group address 16
//                                      different LDS banks at every step of the table
//                                      lookups, and bytes [16/sub * p, 16/sub * (p+1)) of a
//                                      lane belong to ONE scaling group.
//     [lane l][t][p][c]     2 bytes  : binary16 alpha_0..alpha_{q-1} (and the offset if
//                                      present) of (row, block kb) for byte range p of the
//                                      lane, i.e. of scaling sub-group subgroup_of_range(p,
//                                      r, sub); sub = 128/group splits the 128 columns when
//                                      group < 128; the values are replicated when group is
//                                      a larger multiple of 128.
//     When the whole row is one group (group = N, the paper's row-wise parameters) the scales
//     do not depend on the block: the record is stored once per row, [r = 0..15][t][c], and the
//     four lanes 16h + r read the same one (scale_lanes = 16 instead of 64).
//
//   blob = tiles ordered by column slice first, then by row tile, so that a
//   workgroup, which owns one column slice, streams consecutive memory.
//
// Rows >= M and columns >= N are padding: zero bits, zero alpha, zero offset.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define BCQ_HD __host__ __device__
#else
#define BCQ_HD
#endif

namespace bcq {

constexpr int kTileRows = 32;    // rows per tile (two halves of 16)
constexpr int kTileCols = 512;   // columns per tile = per column slice (4 blocks of 128)
constexpr int kBlockCols = 128;  // columns owned by one lane per plane (one 128-bit load)
constexpr int kChunkCols = 8;    // columns per lookup-table index
constexpr int kMaxQ = 4;

struct Geom {
    int M, N, q, z, group;
    int sub;        // scale sub-groups per 128-column block: 128/group for group 32 or 64
                    // (unless the row is one group), else 1
    int nsc;        // binary16 scale entries per (row, block): sub * (q + z)
    int scale_lanes;  // scale records per tile and row half: 64 (one per lane), or 16 (one per row) if group == N
    int Mp, Np;     // padded sizes
    int ntile;      // row tiles   = Mp / 32
    int nslice;     // col slices  = Np / 512
    unsigned tile_plane_bytes;  // 2 * q * 64 * 16
    unsigned tile_bytes;        // plane bytes + 64 * 2 * nsc * 2
};

BCQ_HD inline Geom make_geom(int M, int N, int q, int group, int has_offset)
{
    Geom g;
    g.M = M; g.N = N; g.q = q; g.z = has_offset ? 1 : 0; g.group = group;
    g.sub = (group % kBlockCols == 0 || group == N) ? 1 : kBlockCols / group;
    g.nsc = g.sub * (q + g.z);
    g.Mp = (M + kTileRows - 1) / kTileRows * kTileRows;
    g.Np = (N + kTileCols - 1) / kTileCols * kTileCols;
    g.ntile = g.Mp / kTileRows;
    g.nslice = g.Np / kTileCols;
    g.tile_plane_bytes = 2u * q * 64u * 16u;
    g.scale_lanes = group == N ? 16 : 64;
    g.tile_bytes = g.tile_plane_bytes + (unsigned)g.scale_lanes * 2u * g.nsc * 2u;
    return g;
}

// Which 8-column chunk (0..15) of its 128-column block byte j of lane row r holds, when the
// block is split into `sub` scaling groups (1, 2 or 4).  The high bits (the sub-group) are
// XOR-ed with those of r and the low bits rotated by r: a bijection in j for every r, and in
// r for every j (bank-conflict freedom), that keeps a sub-group in a fixed byte range.
BCQ_HD inline int chunk_of_byte(int j, int r, int sub)
{
    const int lo = 16 / sub - 1, hi = 15 & ~lo;
    return ((j ^ r) & hi) | ((j + r) & lo);
}

// Inverse in j: the byte of lane row r that holds chunk c.
BCQ_HD inline int byte_of_chunk(int c, int r, int sub)
{
    const int lo = 16 / sub - 1, hi = 15 & ~lo;
    return ((c ^ r) & hi) | ((c - r) & lo);
}

// Scaling sub-group (0..sub-1) of the lane's byte range p (bytes [16/sub*p, 16/sub*(p+1))).
BCQ_HD inline int subgroup_of_range(int p, int r, int sub)
{
    return p ^ ((r * sub) >> 4);
}

BCQ_HD inline size_t tile_offset(const Geom &g, int slice, int tile)
{
    return ((size_t)slice * g.ntile + tile) * g.tile_bytes;
}

// Workspace: one 64-bit split-K accumulator word per padded row and batch column.
// Its arrival count has 10 bits, so at most 1023 column slices.
constexpr int kMaxSlices = 1023;

BCQ_HD inline size_t ws_bytes(const Geom &g, int batch)
{
    return g.nslice == 1 ? 0 : (size_t)batch * g.Mp * 8;
}

}  // namespace bcq
