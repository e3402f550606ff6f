// Two activation vectors per call with the GEMV's sign-sum tables (paper Eq. 11 evaluated on the planes, as in
// bcq_gemv.hip), for gfx950.
//
//   y_v[m] = sum_blocks sum_i alpha_i[m,blk] * S_i,v[m,blk]  (+ z[m,blk] * X_v[blk]),   v = 0, 1
//
// Same decomposition as the single-vector kernel -- a workgroup owns one 512-column slice, builds one 256-entry table per
// 8 activations, its waves stream row tiles of the slice and combine the slices with one fixed-point atomic per row,
// slice and vector -- with table entries that hold the sign sums of BOTH vectors side by side (8 bytes, one
// ds_read_b64 per 8 signs serves both).  The tables of a slice are then 128 KB, so a compute unit holds one workgroup;
// it has 16 waves (the registers allow four per SIMD), which keeps as many tiles in flight per compute unit as the
// single-vector kernel's two workgroups of eight.
//
// Table layout: entry p of chunk c (c = 0..63) sits at byte 65536 * (c div 32) + 256 * p + 8 * (c mod 32).  A lane's
// look-up address is one v_perm_b32: byte 0 from a per-lane constant (8 * (c mod 32)), byte 1 the index from the plane
// word, byte 2 from the constant (c div 32, the same for all chunks of a lane's block).  The blob's byte rotation
// makes the 16 lanes of a block read 16 different chunks at every step, so the 32 lanes of a half wave read 32
// different 8-byte columns of a 256-byte bank row.
//
// More vectors do not fit this way (four would need 256 KB, or half slices and twice the atomics): see bcq_lut4.hip
// and bcq_skinny.hip.
#include <atomic>

#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct Gemv2Params {
    const uint8_t *blob;
    const uint16_t *X;  // two rows of activations, ldx apart
    uint16_t *Y;        // two rows of outputs, ldy apart
    unsigned long long *accum;  // [2][Mp] fixed-point row accumulators (value << 10 | arrivals)
    int M, N, Mp, ldx, ldy;
    int ntile, nslice;
    int parts, big_slices;  // slices [0, big_slices) have parts+1 workgroups, the others parts
    unsigned tile_bytes;
    int scale_lane_mask;  // 63: one scale record per lane; 15: one per row (group = N)
};

typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kGemv2Waves = 16;

// One look-up: byte `n` of plane word `w` is the index; `rc` holds the lane's constants for two chunks (bytes 0 and 1:
// 8 * (chunk mod 32)) and its table half (byte 2).  n selects the index byte, k which chunk constant.
template <int n, int k>
__device__ __forceinline__ f32x2 lookup2(const uint8_t *lut, uint32_t w, uint32_t rc)
{
    constexpr uint32_t sel = 0x0c020000u | ((4u + n) << 8) | (uint32_t)k;  // (0, rc.byte2, w.byte n, rc.byte k)
    const uint32_t addr = __builtin_amdgcn_perm(w, rc, sel);
    return *reinterpret_cast<const f32x2 *>(lut + addr);
}

// The 16 look-ups of one (row, block, plane): the sign sums of both vectors over the lane's 128 columns.
__device__ __forceinline__ f32x2 sign_sums2(const uint8_t *lut, const u32x4 &p, const uint32_t (&rc)[8])
{
    f32x2 d[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        f32x2 a = lookup2<0, 0>(lut, p[v], rc[2 * v]);
        a += lookup2<1, 1>(lut, p[v], rc[2 * v]);
        a += lookup2<2, 0>(lut, p[v], rc[2 * v + 1]);
        a += lookup2<3, 1>(lut, p[v], rc[2 * v + 1]);
        d[v] = a;
    }
    return (d[0] + d[1]) + (d[2] + d[3]);
}

__device__ __forceinline__ void complete_row2(const Gemv2Params &p, int v, int row, unsigned long long total)
{
    if (arrivals_of(total) == (unsigned)p.nslice) {
        if (row < p.M) p.Y[(size_t)v * p.ldy + row] = float_to_half_bits(decode_total(total));
        __hip_atomic_store(p.accum + (size_t)v * p.Mp + row, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int Q, int Z>
__global__ __launch_bounds__(kGemv2Waves * 64) void bcq_gemv2_kernel(Gemv2Params p)
{
    constexpr int NW = kGemv2Waves;
    __shared__ __attribute__((aligned(16))) uint8_t lut[2 * 65536];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int slice, part, parts;
    {
        const int big_groups = p.big_slices * (p.parts + 1);
        if ((int)blockIdx.x < big_groups) {
            parts = p.parts + 1;
            slice = blockIdx.x / parts;
            part = blockIdx.x - slice * parts;
        } else {
            parts = p.parts;
            const int rest = blockIdx.x - big_groups;
            slice = p.big_slices + rest / parts;
            part = rest - (rest / parts) * parts;
        }
    }
    // Row tiles of this workgroup: an even split of the slice's tiles over its workgroups; wave w takes the tiles
    // first + w, first + w + NW, ... (the workgroup streams NW neighbouring tiles at a time).
    const int g_begin = (int)(((long long)part * p.ntile) / parts);
    const int t_end = (int)(((long long)(part + 1) * p.ntile) / parts);
    const int t_begin = g_begin + wave < t_end ? g_begin + wave : t_end;
    const uint8_t *tile_ptr = p.blob + ((size_t)slice * p.ntile + t_begin) * p.tile_bytes;

    // the first tile's loads are started before the tables are built
    TileRegs<Q, Z, 1> cur;
    const int col0 = slice * kTileCols + kChunkCols * lane;  // lane = chunk
    u32x4 xr[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if (col0 < p.N) {
        xr[0] = *reinterpret_cast<const u32x4 *>(p.X + col0);
        xr[1] = *reinterpret_cast<const u32x4 *>(p.X + (size_t)p.ldx + col0);
    }
    if (t_begin < t_end) load_tile<Q, Z, 1>(cur, tile_ptr, lane, lane & p.scale_lane_mask);

    // ---- sign-sum tables for the 512 activations of this slice, both vectors ----------------
    {
        f32x2 xv[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xv[2 * e] = f32x2{half_bits_to_float(xr[0][e] & 0xffffu), half_bits_to_float(xr[1][e] & 0xffffu)};
            xv[2 * e + 1] = f32x2{half_bits_to_float(xr[0][e] >> 16), half_bits_to_float(xr[1][e] >> 16)};
        }
        constexpr int IPW = 256 / NW;  // indices built by one wave: 16, i.e. bits 4..7 of the index are the wave
        f32x2 hi = {0.0f, 0.0f};
#pragma unroll
        for (int b = 4; b < 8; ++b) hi += ((wave >> (b - 4)) & 1) ? xv[b] : -xv[b];
        f32x2 lo[8];
#pragma unroll
        for (int a = 0; a < 8; ++a)
            lo[a] = ((a & 1) ? xv[0] : -xv[0]) + ((a & 2) ? xv[1] : -xv[1]) + ((a & 4) ? xv[2] : -xv[2]);
        uint8_t *dst = lut + 65536 * (lane >> 5) + 8 * (lane & 31);
#pragma unroll
        for (int m = 0; m < IPW / 8; ++m) {
            const f32x2 mid = hi + ((m & 1) ? xv[3] : -xv[3]);
#pragma unroll
            for (int a = 0; a < 8; ++a) *reinterpret_cast<f32x2 *>(dst + 256 * (wave * IPW + m * 8 + a)) = lo[a] + mid;
        }
    }
    __syncthreads();

    // ---- per-lane constants ----------------------------------------------------
    const int r = lane & 15, h = lane >> 4;
    uint32_t rc[8];  // rc[2v + k]: bytes 0, 1 = 8 * (chunk mod 32) of the lane's bytes 4v + 2k, 4v + 2k + 1; byte 2 = table half
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int c0 = 16 * h + chunk_of_byte(4 * v + 2 * k, r, 1), c1 = 16 * h + chunk_of_byte(4 * v + 2 * k + 1, r, 1);
            rc[2 * v + k] = (uint32_t)(8 * (c0 & 31)) | ((uint32_t)(8 * (c1 & 31)) << 8) | ((uint32_t)(h >> 1) << 16);
        }
    f32x2 xsum = {0.0f, 0.0f};  // sums of the activations of this lane's block
    if (Z) {
#pragma unroll
        for (int c = 0; c < 16; ++c)
            xsum += *reinterpret_cast<const f32x2 *>(lut + 65536 * (h >> 1) + 256 * 255 + 8 * ((16 * h + c) & 31));
    }

    // ---- stream the row tiles; the split-K atomics are pipelined as in the single-vector kernel: an iteration
    // waits for its tile (and with it for the atomics issued one iteration earlier), completes the rows of tile
    // k-2, issues the atomics of tile k-1, requests tile k+1 and computes tile k ----
    const bool split_k = p.nslice > 1;
    // After the lane swaps the sums of rows 0..15 sit in the lanes 0..15 AND 16..31, those of rows 16..31 in the lanes
    // 32..47 AND 48..63.  The first copy reports vector 0, the second vector 1: one atomic (or store) instruction of 64
    // lanes per tile instead of two of 32.
    const int vec = (lane >> 4) & 1;                       // the vector this lane reports
    const int rep_row = (lane & 15) | ((lane >> 5) << 4);  // its row inside the tile
    unsigned long long *const accum = p.accum + (size_t)vec * p.Mp;
    int held_tile = -1;
    float held = 0.0f;
    int pend_tile = -1;
    unsigned long long pend_old = 0, pend_mine = 0;

    for (int tile = t_begin; tile < t_end; tile += NW) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (split_k) {
            if (pend_tile >= 0) complete_row2(p, vec, pend_tile * kTileRows + rep_row, pend_old + pend_mine);
            pend_tile = held_tile;
            if (held_tile >= 0) {
                pend_mine = encode_partial_f32(held);
                pend_old = __hip_atomic_fetch_add(accum + held_tile * kTileRows + rep_row, pend_mine, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        TileRegs<Q, Z, 1> nxt;
        tile_ptr += (size_t)NW * p.tile_bytes;
        if (tile + NW < t_end) load_tile<Q, Z, 1>(nxt, tile_ptr, lane, lane & p.scale_lane_mask);

        f32x2 acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x2 a = {0.0f, 0.0f};
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                const f32x2 ss = sign_sums2(lut, cur.planes[t][i], rc);
                const float alpha = scale_of<Q, Z, 1>(cur, t, 0, i);
                a[0] = fmaf(alpha, ss[0], a[0]);
                a[1] = fmaf(alpha, ss[1], a[1]);
            }
            if (Z) {
                const float z = scale_of<Q, Z, 1>(cur, t, 0, Q);
                a[0] = fmaf(z, xsum[0], a[0]);
                a[1] = fmaf(z, xsum[1], a[1]);
            }
            acc[t] = a;
        }
        const float out0 = sum_block_owners(acc[0][0], acc[1][0]), out1 = sum_block_owners(acc[0][1], acc[1][1]);
        const float out = vec ? out1 : out0;
        if (split_k) {
            held = out;
            held_tile = tile;
        } else {
            const int row = tile * kTileRows + rep_row;
            if (row < p.M) p.Y[(size_t)vec * p.ldy + row] = float_to_half_bits(out);
        }
        if (tile + NW < t_end) cur = nxt;
    }

    if (split_k) {  // drain: two tiles may still be in the pipeline
        if (held_tile >= 0) {
            const unsigned long long mine = encode_partial_f32(held);
            const unsigned long long old = __hip_atomic_fetch_add(accum + held_tile * kTileRows + rep_row, mine,
                                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (pend_tile >= 0) complete_row2(p, vec, pend_tile * kTileRows + rep_row, pend_old + pend_mine);
            complete_row2(p, vec, held_tile * kTileRows + rep_row, old + mine);
        } else if (pend_tile >= 0) {
            complete_row2(p, vec, pend_tile * kTileRows + rep_row, pend_old + pend_mine);
        }
    }
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
// Workgroups of the kernel the current device holds at once (128 KB of LDS: one per compute unit).
static int gemv2_resident_groups()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int groups = cached[dev].load(std::memory_order_relaxed);
    if (groups == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bcq_gemv2_kernel<3, 0>, kGemv2Waves * 64, 0) != hipSuccess ||
            per_cu < 1)
            per_cu = 1;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        groups = per_cu * cus;
        cached[dev].store(groups, std::memory_order_relaxed);
    }
    return groups;
}

template <int Q, int Z>
static hipError_t launch_gemv2_qz(const Gemv2Params &p, int groups, hipStream_t stream)
{
    hipLaunchKernelGGL((bcq_gemv2_kernel<Q, Z>), dim3((unsigned)groups), dim3(kGemv2Waves * 64), 0, stream, p);
    return hipGetLastError();
}

bool gemv2_applies(const Geom &g, int batch, const void *workspace)
{
    // one scaling group per block; split-K accumulators unless the layer is a single slice
    return batch == 2 && g.sub == 1 && (workspace != nullptr || g.nslice == 1);
}

hipError_t launch_gemv2(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy,
                        void *workspace, const GemvTuning &tuning, hipStream_t stream)
{
    if (!gemv2_applies(g, 2, workspace)) return hipErrorInvalidValue;
    // as many workgroups as the device holds, at least one per slice, at most one per row tile of a slice
    const long long tiles = (long long)g.nslice * g.ntile;
    long long groups = tuning.workgroups > 0 ? tuning.workgroups : gemv2_resident_groups();
    const long long busy = (tiles + kGemv2Waves - 1) / kGemv2Waves;  // every wave a tile
    if (tuning.workgroups <= 0 && groups > busy) groups = busy;
    if (groups < g.nslice) groups = g.nslice;
    if (groups > tiles) groups = tiles;
    Gemv2Params p;
    p.parts = (int)(groups / g.nslice);
    p.big_slices = (int)(groups % g.nslice);
    p.blob = static_cast<const uint8_t *>(packed);
    p.X = X; p.Y = Y;
    p.accum = static_cast<unsigned long long *>(workspace);
    p.M = g.M; p.N = g.N; p.Mp = g.Mp; p.ldx = ldx; p.ldy = ldy;
    p.ntile = g.ntile; p.nslice = g.nslice;
    p.tile_bytes = g.tile_bytes;
    p.scale_lane_mask = g.scale_lanes - 1;
    switch (g.q * 2 + g.z) {
        case 2: return launch_gemv2_qz<1, 0>(p, (int)groups, stream);
        case 3: return launch_gemv2_qz<1, 1>(p, (int)groups, stream);
        case 4: return launch_gemv2_qz<2, 0>(p, (int)groups, stream);
        case 5: return launch_gemv2_qz<2, 1>(p, (int)groups, stream);
        case 6: return launch_gemv2_qz<3, 0>(p, (int)groups, stream);
        case 7: return launch_gemv2_qz<3, 1>(p, (int)groups, stream);
        case 8: return launch_gemv2_qz<4, 0>(p, (int)groups, stream);
        case 9: return launch_gemv2_qz<4, 1>(p, (int)groups, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace bcq
