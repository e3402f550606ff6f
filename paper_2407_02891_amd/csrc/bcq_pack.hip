// bcq_pack / bcq_unpack kernels: canonical operands of Eq. 11 (per-weight codes,
// alpha[M][G][q], offset[M][G]) <-> the tiled blob described in bcq_layout.h.
// Offline step; written for clarity, not speed.
#include "bcq_internal.h"

namespace bcq {

// A pack call covers the rows [row0, row0 + rows) of the layer; the call that reaches the last
// row also writes the padding rows.  `codes`, `alpha`, `offset` hold only the covered rows.
__device__ __forceinline__ bool row_is_mine(const Geom &g, int row, int row0, int rows)
{
    return row >= row0 && (row < row0 + rows || (row >= g.M && row0 + rows == g.M));
}

__global__ void pack_planes_kernel(Geom g, int row0, int rows, const uint8_t *__restrict__ codes,
                                   uint8_t *__restrict__ blob, size_t total_dwords)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total_dwords) return;
    const unsigned dwords_per_tile = g.tile_plane_bytes / 4;
    size_t tile_lin = gid / dwords_per_tile;
    unsigned rem = (unsigned)(gid % dwords_per_tile);
    int slice = (int)(tile_lin / g.ntile), tile = (int)(tile_lin % g.ntile);
    int d = rem & 3, lane = (rem >> 2) & 63, ti = rem >> 8;
    int t = ti / g.q, i = ti % g.q;
    int r = lane & 15, h = lane >> 4;
    int row = kTileRows * tile + 16 * t + r;
    int kb = 4 * slice + h;
    if (!row_is_mine(g, row, row0, rows)) return;
    uint32_t word = 0;
    if (row < g.M) {
        for (int n = 0; n < 4; ++n) {
            int j = 4 * d + n;
            int c = chunk_of_byte(j, r, g.sub);
            int col = kBlockCols * kb + kChunkCols * c;
            if (col < g.N) {
                const uint8_t *src = codes + (size_t)(row - row0) * g.N + col;
                for (int b = 0; b < 8; ++b)
                    word |= (uint32_t)((src[b] >> i) & 1) << (8 * n + b);
            }
        }
    }
    uint32_t *dst = reinterpret_cast<uint32_t *>(blob + tile_offset(g, slice, tile) +
                                                 ((size_t)(ti * 64 + lane) * 16 + 4 * d));
    *dst = word;
}

__global__ void pack_scales_kernel(Geom g, int row0, int rows, const uint16_t *__restrict__ alpha,
                                   const uint16_t *__restrict__ offset,
                                   uint8_t *__restrict__ blob, size_t total_entries)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total_entries) return;
    const unsigned per_tile = (unsigned)g.scale_lanes * 2u * g.nsc;  // with 16 records per half tile, `lane` below is the row
    size_t tile_lin = gid / per_tile;
    unsigned e = (unsigned)(gid % per_tile);
    int slice = (int)(tile_lin / g.ntile), tile = (int)(tile_lin % g.ntile);
    int lane = e / (2 * g.nsc), rr = e % (2 * g.nsc);
    int t = rr / g.nsc, sc = rr % g.nsc;
    int qz = g.q + g.z;
    int range = sc / qz, c = sc % qz;
    int r = lane & 15, h = lane >> 4;
    int row = kTileRows * tile + 16 * t + r;
    if (!row_is_mine(g, row, row0, rows)) return;
    int col = kBlockCols * (4 * slice + h) + subgroup_of_range(range, r, g.sub) * (kBlockCols / g.sub);
    uint16_t val = 0;
    if (row < g.M && col < g.N) {
        size_t G = g.N / g.group, grp = col / g.group, src_row = row - row0;
        val = c < g.q ? alpha[(src_row * G + grp) * g.q + c] : offset[src_row * G + grp];
    }
    uint16_t *dst = reinterpret_cast<uint16_t *>(blob + tile_offset(g, slice, tile) +
                                                 g.tile_plane_bytes + (size_t)e * 2);
    *dst = val;
}

__global__ void unpack_codes_kernel(Geom g, const uint8_t *__restrict__ blob,
                                    uint8_t *__restrict__ codes)
{
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (size_t)g.M * g.N) return;
    int row = (int)(gid / g.N), col = (int)(gid % g.N);
    int slice = col / kTileCols, h = (col % kTileCols) / kBlockCols;
    int c = (col % kBlockCols) / kChunkCols, bit = col % kChunkCols;
    int tile = row / kTileRows, t = (row % kTileRows) / 16, r = row % 16;
    int j = byte_of_chunk(c, r, g.sub);
    const uint8_t *base = blob + tile_offset(g, slice, tile);
    uint8_t code = 0;
    for (int i = 0; i < g.q; ++i) {
        uint8_t byte = base[(size_t)((t * g.q + i) * 64 + 16 * h + r) * 16 + j];
        code |= (uint8_t)(((byte >> bit) & 1) << i);
    }
    codes[gid] = code;
}

__global__ void unpack_scales_kernel(Geom g, const uint8_t *__restrict__ blob,
                                     uint16_t *__restrict__ alpha, uint16_t *__restrict__ offset)
{
    size_t G = g.N / g.group;
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (size_t)g.M * G) return;
    int row = (int)(gid / G);
    int col = (int)(gid % G) * g.group;           // first column of the group
    int slice = col / kTileCols, h = (col % kTileCols) / kBlockCols;
    int tile = row / kTileRows, t = (row % kTileRows) / 16, r = row % 16;
    // subgroup_of_range is its own inverse in its first argument
    int range = subgroup_of_range((col % kBlockCols) / (kBlockCols / g.sub), r, g.sub);
    int lane = (16 * h + r) & (g.scale_lanes - 1), qz = g.q + g.z;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(
        blob + tile_offset(g, slice, tile) + g.tile_plane_bytes) +
        (size_t)lane * 2 * g.nsc + (size_t)t * g.nsc + (size_t)range * qz;
    if (alpha)
        for (int c = 0; c < g.q; ++c) alpha[gid * g.q + c] = src[c];
    if (offset && g.z) offset[gid] = src[g.q];
}

__global__ void fill_zero_kernel(uint32_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

static unsigned blocks_for(size_t n, unsigned threads)
{
    return (unsigned)((n + threads - 1) / threads);
}

hipError_t launch_pack(const Geom &g, int row0, int rows, const uint8_t *codes, const uint16_t *alpha,
                       const uint16_t *offset, void *packed, hipStream_t stream)
{
    size_t tiles = (size_t)g.nslice * g.ntile;
    size_t nd = tiles * (g.tile_plane_bytes / 4);
    size_t ne = tiles * (size_t)g.scale_lanes * 2u * g.nsc;
    hipLaunchKernelGGL(pack_planes_kernel, dim3(blocks_for(nd, 256)), dim3(256), 0, stream, g, row0, rows,
                       codes, static_cast<uint8_t *>(packed), nd);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(pack_scales_kernel, dim3(blocks_for(ne, 256)), dim3(256), 0, stream, g, row0, rows,
                       alpha, offset, static_cast<uint8_t *>(packed), ne);
    return hipGetLastError();
}

hipError_t launch_unpack(const Geom &g, const void *packed, uint8_t *codes, uint16_t *alpha,
                         uint16_t *offset, hipStream_t stream)
{
    const uint8_t *blob = static_cast<const uint8_t *>(packed);
    if (codes) {
        size_t n = (size_t)g.M * g.N;
        hipLaunchKernelGGL(unpack_codes_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, stream, g,
                           blob, codes);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (alpha || offset) {
        size_t n = (size_t)g.M * (g.N / g.group);
        hipLaunchKernelGGL(unpack_scales_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, stream, g,
                           blob, alpha, offset);
    }
    return hipGetLastError();
}

hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t stream)
{
    size_t n = bytes / 4;
    if (n == 0) return hipSuccess;
    unsigned blocks = blocks_for(n, 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream,
                       static_cast<uint32_t *>(ptr), n);
    return hipGetLastError();
}

}  // namespace bcq
