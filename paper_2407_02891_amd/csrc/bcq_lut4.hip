// Binary-coding product for 2..4 activation vectors on gfx950 with sign-sum tables (paper Eq. 11 applied to
// up to four vectors at once), reading the packed weights ONCE.
//
// The batch-1 GEMV (bcq_gemv.hip) looks up, for every 8 signs, the signed sum of 8 activations in a 256-entry
// table.  Here a table entry holds that sum for FOUR activation vectors side by side (16 bytes), so one
// ds_read_b128 serves all of them: the work per weight bit is one LDS read and four additions whatever the
// batch, against one matrix-core operand per 8 signs in the skinny GEMM kernel (bcq_skinny.hip), which is
// bound by delivering those operands.  The price is the table size: 16 bytes x 256 patterns x 32 chunks = 128 KB
// hold the tables of HALF a column slice (256 columns), and with split-K per half slice every row would need
// 2 nslice x batch atomics.  So the loop nest is turned round: a workgroup keeps a set of rows, walks along K
// and rebuilds the tables for every half slice (120 vector-ALU instructions per thread), while the partial sums
// stay in registers; rows are flushed when the workgroup's range of work leaves them.
//
//  * Workgroup: 16 waves (128 registers each), one per CU (LDS).  A work unit is (row group of 32 row tiles, half slice): wave w takes
//    the tiles 2w and 2w+1 of the group, lanes 0..31 the first, lanes 32..63 the second; lane 16 h' + r of a half
//    holds (row r, block 2 half + h') of its tile, exactly the blob's lane 32 half + 16 h' + r (bcq_layout.h).
//    The units, row group first, are cut into equal contiguous ranges, one per workgroup; the workgroups that share
//    a row group are combined with the fixed-point split-K atomics of the GEMV (bcq_device.h).
//  * Table layout: entry (chunk c, pattern p) at byte p * 512 + c * 16.  Byte j of a lane's 16 bytes is chunk
//    (j + r) mod 16 of its block (the blob's rotation), so the 16 lanes that a ds_read_b128 serves together
//    (lanes {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31}, +32: 16 different r) read 16 different
//    16-byte columns of the 256-byte bank row: no conflicts.
//  * Loads of the next unit's sign planes go through one buffer descriptor over the whole blob (offsets of
//    tiles that do not exist are out of range and return zeros), requested before the current unit's look-ups;
//    its activations are fetched by the first two waves and parked in LDS.
#include <atomic>

#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct Lut4Params {
    const uint8_t *blob;
    const uint16_t *X;
    uint16_t *Y;
    unsigned long long *accum;  // [batch][Mp]
    int M, N, Mp, batch, ldx, ldy;
    int ntile, nslice;
    int nrg;    // row groups of 32 tiles
    int units;  // nrg * 2 * nslice
    unsigned tile_bytes, blob_bytes;
    int scale_lane_mask;  // 63: one scale record per lane; 15: one per row (group = N)
};

constexpr int kLutWaves = 16;
constexpr int kLutTilesPerGroup = 2 * kLutWaves;
constexpr int kHalfCols = kTileCols / 2;  // 256
constexpr uint32_t kLutNoTile = 0xfff00000u;  // offset of "no such tile"; blobs must be smaller

// Byte offset in the blob of (slice, tile), or of "no such tile": beyond every blob this kernel accepts and far
// enough from 2^32 for the offsets added to it not to wrap, so that the loads return zeros.
__device__ __forceinline__ uint32_t lut_tile_base(const Lut4Params &p, int slice, int tile, bool wanted)
{
    return (wanted && tile < p.ntile) ? (uint32_t)(((size_t)slice * p.ntile + tile) * p.tile_bytes) : kLutNoTile;
}

// Sign plane k (row half k div Q, plane k mod Q) of this lane; blob_lane = 32 half + 16 h' + r.
__device__ __forceinline__ u32x4 lut_load_plane(__amdgpu_buffer_rsrc_t blob, uint32_t base, uint32_t blob_lane, int k)
{
    return __builtin_amdgcn_raw_buffer_load_b128(blob, base + 1024u * k + 16u * blob_lane, 0, 2 /* non-temporal */);
}

template <int Q, int Z>
__device__ __forceinline__ void lut_load_scales(uint32_t (&sc)[Q + Z], __amdgpu_buffer_rsrc_t blob, const Lut4Params &p,
                                                uint32_t base, uint32_t blob_lane)
{
    const uint32_t so = base + 2u * Q * 1024u + 4u * (Q + Z) * (blob_lane & (uint32_t)p.scale_lane_mask);
#pragma unroll
    for (int c = 0; c < Q + Z; ++c) sc[c] = __builtin_amdgcn_raw_buffer_load_b32(blob, so + 4u * c, 0, 2);
}

template <int Q, int Z>
__global__ __launch_bounds__(64 * kLutWaves) void bcq_lut4_kernel(Lut4Params p)
{
    __shared__ __attribute__((aligned(16))) uint8_t tab[32 * 256 * 16];      // 128 KB
    __shared__ __attribute__((aligned(16))) uint16_t xstage[4 * kHalfCols];  // 2 KB: [vector][column of the half slice]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (the longer ranges spread evenly over the workgroups: placed on the first ones, whose ranges are neighbours in
    // memory, they cost 2 to 3 us on the layers with five or six units per workgroup)
    const int groups = gridDim.x;
    const int u_begin = first_unit<false>(blockIdx.x, p.units, groups, 0, 0);
    const int u_end = first_unit<false>(blockIdx.x + 1, p.units, groups, 0, 0);
    if (u_begin >= u_end) return;  // uniform for the workgroup, before any barrier
    const int nh = 2 * p.nslice;   // half slices per row group

    const int bl = lane & 31;          // lane inside its half of the wave = 16 h' + r
    const int r = lane & 15;
    const int hq = (lane >> 4) & 1;    // h': block inside the half slice
    const int which = lane >> 5;       // first or second tile of the wave's pair
    uint32_t col_bytes[16];            // byte offset of the chunk that byte j of this lane addresses, inside a pattern's 512 bytes
#pragma unroll
    for (int j = 0; j < 16; ++j) col_bytes[j] = 16u * (16 * hq + ((j + r) & 15));

    const __amdgpu_buffer_rsrc_t blob = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.blob), 0, (int)p.blob_bytes, kRawBufferFlags);
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.X), 0, (int)(2u * (uint32_t)p.batch * (uint32_t)p.ldx), kRawBufferFlags);
    // activations of a half slice: thread (vector v = tid / 32, chunk c = tid % 32) of the first two waves fetches 8 values
    auto x_fetch = [&](int hs, bool wanted) -> u32x4 {
        const int v = tid >> 5, c = tid & 31;
        const int col = (hs >> 1) * kTileCols + (hs & 1) * kHalfCols + kChunkCols * c;
        const bool ok = wanted && tid < 128 && v < p.batch && col < p.N;
        const uint32_t off = ok ? 2u * ((uint32_t)v * (uint32_t)p.ldx + (uint32_t)col) : 0xfffffff0u;
        return __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0);
    };
    auto x_park = [&](const u32x4 &xr) {
        if (tid < 128) *reinterpret_cast<u32x4 *>(xstage + (tid >> 5) * kHalfCols + (tid & 31) * kChunkCols) = xr;
    };

    int rg = u_begin / nh, hs = u_begin - rg * nh;
    TileRegs<Q, Z, 1> cur;
    {
        const uint32_t base = lut_tile_base(p, hs >> 1, kLutTilesPerGroup * rg + 2 * wave + which, true);
#pragma unroll
        for (int k = 0; k < 2 * Q; ++k) cur.planes[k / Q][k % Q] = lut_load_plane(blob, base, 32u * (hs & 1) + bl, k);
        lut_load_scales<Q, Z>(cur.scales, blob, p, base, 32u * (hs & 1) + bl);
    }
    x_park(x_fetch(hs, true));
    __syncthreads();

    int u = u_begin;
    while (u < u_end) {
        // one segment: the units of this workgroup that belong to row group `rg`
        const int seg_end = min(u_end, (rg + 1) * nh);
        const int seg_rg = rg;
        float acc[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][v] = 0.0f;
        for (; u < seg_end; ++u) {
            // ---- tables of this half slice: thread (chunk c, patterns 8 pg .. 8 pg + 7), four vectors side by side
#pragma unroll
            for (int pp = 0; pp < 32 / (2 * kLutWaves); ++pp) {
                const int c = tid & 31, pg = (tid >> 5) + 2 * kLutWaves * pp;
                f32x4 e[8];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const u32x4 xr = *reinterpret_cast<const u32x4 *>(xstage + v * kHalfCols + c * kChunkCols);
                    float xv[8];
                    xv[0] = half_bits_to_float(xr.x & 0xffffu); xv[1] = half_bits_to_float(xr.x >> 16);
                    xv[2] = half_bits_to_float(xr.y & 0xffffu); xv[3] = half_bits_to_float(xr.y >> 16);
                    xv[4] = half_bits_to_float(xr.z & 0xffffu); xv[5] = half_bits_to_float(xr.z >> 16);
                    xv[6] = half_bits_to_float(xr.w & 0xffffu); xv[7] = half_bits_to_float(xr.w >> 16);
                    float hi = 0.0f;  // bits 3..7 of the pattern are pg
#pragma unroll
                    for (int b = 3; b < 8; ++b) hi += ((pg >> (b - 3)) & 1) ? xv[b] : -xv[b];
#pragma unroll
                    for (int a = 0; a < 8; ++a)
                        e[a][v] = (((a & 1) ? xv[0] : -xv[0]) + ((a & 2) ? xv[1] : -xv[1]) + ((a & 4) ? xv[2] : -xv[2])) + hi;
                }
#pragma unroll
                for (int a = 0; a < 8; ++a) *reinterpret_cast<f32x4 *>(tab + (size_t)(8 * pg + a) * 512 + 16 * c) = e[a];
            }
            __syncthreads();  // tables complete; everyone has read the parked activations

            // ---- requests for the next unit of this workgroup (it may be the first of the next segment): its
            // activations and scales now, each of its sign planes as soon as the current one is used up, into the
            // same registers -- every plane then has a whole unit to arrive, and no second tile is held
            const bool more = u + 1 < u_end;
            int n_hs = hs + 1, n_rg = rg;
            if (n_hs == nh) { n_hs = 0; n_rg = rg + 1; }
            const u32x4 n_x = x_fetch(n_hs, more);
            const uint32_t n_base = lut_tile_base(p, n_hs >> 1, kLutTilesPerGroup * n_rg + 2 * wave + which, more);
            const uint32_t n_lane = 32u * (n_hs & 1) + bl;
            uint32_t n_scales[Q + Z];
            lut_load_scales<Q, Z>(n_scales, blob, p, n_base, n_lane);

            // ---- look-ups: for every (row half, plane) 16 table entries of four sums each
            float xsum[4] = {0.f, 0.f, 0.f, 0.f};  // sums of the block's activations: the entries of pattern 255
            if (Z) {
#pragma unroll
                for (int c0 = 0; c0 < 16; c0 += 4) {
                    f32x4 e[4];
#pragma unroll
                    for (int n = 0; n < 4; ++n) e[n] = *reinterpret_cast<const f32x4 *>(tab + 255 * 512 + 16 * (16 * hq + c0 + n));
                    const f32x4 g = (e[0] + e[1]) + (e[2] + e[3]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) xsum[v] += g[v];
                    asm volatile("" : "+v"(xsum[0]), "+v"(xsum[1]), "+v"(xsum[2]), "+v"(xsum[3]));  // (registers, as below)
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    const u32x4 w = cur.planes[t][i];
                    float s4[4] = {0.f, 0.f, 0.f, 0.f};
                    constexpr int kDwords = (Q + Z <= 3) ? 2 : 1;  // look-ups in flight: 8, or 4 where registers are short
#pragma unroll
                    for (int d = 0; d < 4; d += kDwords) {
                        f32x4 e[4 * kDwords];
#pragma unroll
                        for (int n = 0; n < 4 * kDwords; ++n) {
                            const uint32_t byte = (w[d + (n >> 2)] >> (8 * (n & 3))) & 0xffu;
                            e[n] = *reinterpret_cast<const f32x4 *>(tab + ((byte << 9) | col_bytes[4 * d + n]));
                        }
                        f32x4 g = (e[0] + e[1]) + (e[2] + e[3]);
                        if (kDwords == 2) g += (e[4 * kDwords - 4] + e[4 * kDwords - 3]) + (e[4 * kDwords - 2] + e[4 * kDwords - 1]);
#pragma unroll
                        for (int v = 0; v < 4; ++v) s4[v] += g[v];
                        // the sums have to exist here: otherwise every look-up of the unit is requested before the
                        // first addition and their results do not fit the registers
                        asm volatile("" : "+v"(s4[0]), "+v"(s4[1]), "+v"(s4[2]), "+v"(s4[3]));
                    }
                    const float alpha = scale_of<Q, Z, 1>(cur, t, 0, i);
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[t][v] = fmaf(alpha, s4[v], acc[t][v]);
                    cur.planes[t][i] = lut_load_plane(blob, n_base, n_lane, t * Q + i);  // the next unit's, zeros if none
                }
                if (Z) {
                    const float z = scale_of<Q, Z, 1>(cur, t, 0, Q);
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[t][v] = fmaf(z, xsum[v], acc[t][v]);
                }
            }
#pragma unroll
            for (int c = 0; c < Q + Z; ++c) cur.scales[c] = n_scales[c];
            x_park(n_x);  // (after the barrier above: nobody reads the old ones any more)
            rg = n_rg; hs = n_hs;
            __syncthreads();  // everyone done with these tables; next activations parked
        }
        // ---- this workgroup is done with the row group: combine the two blocks of a row, then flush
        const int arrivals = owner_of_unit<false>((seg_rg + 1) * nh - 1, p.units, groups, 0, 0) -
                             owner_of_unit<false>(seg_rg * nh, p.units, groups, 0, 0) + 1;
        // (the lane index is passed through an empty asm so that the per-lane address arithmetic of the flush is
        // not hoisted out of the outer loop into registers that stay live during the units)
        int flush_lane = lane;
        asm volatile("" : "+v"(flush_lane));
        const int f_r = flush_lane & 15, f_hq = (flush_lane >> 4) & 1;
        const int tile = kLutTilesPerGroup * seg_rg + 2 * wave + (flush_lane >> 5);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][v] += __shfl_xor(acc[t][v], 16);  // lanes 16 h' + r, h' = 0, 1
        if (f_hq == 0 && tile < p.ntile) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int row = tile * kTileRows + 16 * t + f_r;
                if (arrivals == 1) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (v < p.batch && row < p.M) p.Y[(size_t)v * p.ldy + row] = float_to_half_bits(acc[t][v]);
                } else {
                    unsigned long long mine[4], old[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        mine[v] = encode_partial(acc[t][v]);
                        old[v] = 0;
                        if (v < p.batch)
                            old[v] = __hip_atomic_fetch_add(p.accum + (size_t)v * p.Mp + row, mine[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const unsigned long long total = old[v] + mine[v];
                        if (v < p.batch && arrivals_of(total) == (unsigned)arrivals) {
                            if (row < p.M) p.Y[(size_t)v * p.ldy + row] = float_to_half_bits(decode_total(total));
                            __hip_atomic_store(p.accum + (size_t)v * p.Mp + row, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
        }
    }
}

// Workgroups of the kernel the current device holds at once (128 KB of LDS: one per compute unit).
static int lut4_resident_groups()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int groups = cached[dev].load(std::memory_order_relaxed);
    if (groups == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bcq_lut4_kernel<3, 0>, 64 * kLutWaves, 0) != hipSuccess || per_cu < 1)
            per_cu = 1;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        groups = per_cu * cus;
        cached[dev].store(groups, std::memory_order_relaxed);
    }
    return groups;
}

template <int Q, int Z>
static hipError_t launch_lut4_qz(const Lut4Params &p, int groups, hipStream_t stream)
{
    hipLaunchKernelGGL((bcq_lut4_kernel<Q, Z>), dim3((unsigned)groups), dim3(64 * kLutWaves), 0, stream, p);
    return hipGetLastError();
}

bool lut4_applies(const Geom &g, int batch, const void *workspace)
{
    // one scaling group per block; split-K accumulators needed (two half slices may go to two workgroups); the whole
    // blob must be addressable through one buffer descriptor (32-bit offsets)
    const unsigned long long blob_bytes = (unsigned long long)g.nslice * g.ntile * g.tile_bytes;
    // (four planes plus offset do not fit the 128 registers of a 16-wave workgroup)
    return batch >= 2 && batch <= 4 && g.sub == 1 && g.nslice >= 2 && !(g.q == 4 && g.z) && workspace != nullptr &&
           blob_bytes < kLutNoTile;
}

hipError_t launch_lut4(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy, int batch,
                       void *workspace, const GemvTuning &tuning, hipStream_t stream)
{
    if (!lut4_applies(g, batch, workspace)) return hipErrorInvalidValue;
    Lut4Params p;
    p.blob = static_cast<const uint8_t *>(packed);
    p.X = X; p.Y = Y;
    p.accum = static_cast<unsigned long long *>(workspace);
    p.M = g.M; p.N = g.N; p.Mp = g.Mp; p.batch = batch; p.ldx = ldx; p.ldy = ldy;
    p.ntile = g.ntile; p.nslice = g.nslice;
    p.nrg = (g.ntile + kLutTilesPerGroup - 1) / kLutTilesPerGroup;
    const long long units = (long long)p.nrg * 2 * g.nslice;
    if (units > 0x7fffffffLL) return hipErrorInvalidValue;
    p.units = (int)units;
    p.tile_bytes = g.tile_bytes;
    p.blob_bytes = (unsigned)((unsigned long long)g.nslice * g.ntile * g.tile_bytes);
    p.scale_lane_mask = g.scale_lanes - 1;
    long long groups = tuning.workgroups > 0 ? tuning.workgroups : lut4_resident_groups();
    if (groups > units) groups = units;
    if (groups < 1) groups = 1;
    switch (g.q * 2 + g.z) {
        case 2: return launch_lut4_qz<1, 0>(p, (int)groups, stream);
        case 3: return launch_lut4_qz<1, 1>(p, (int)groups, stream);
        case 4: return launch_lut4_qz<2, 0>(p, (int)groups, stream);
        case 5: return launch_lut4_qz<2, 1>(p, (int)groups, stream);
        case 6: return launch_lut4_qz<3, 0>(p, (int)groups, stream);
        case 7: return launch_lut4_qz<3, 1>(p, (int)groups, stream);
        case 8: return launch_lut4_qz<4, 0>(p, (int)groups, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace bcq
