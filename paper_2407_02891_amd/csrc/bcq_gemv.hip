// Batch-1 binary-coding GEMV for gfx950 (paper Eq. 11 evaluated on the planes).
//
//   y[m] = sum_blocks sum_i alpha_i[m,blk] * S_i[m,blk]  (+ z[m,blk] * X[blk])
//   S_i[m,blk] = sum_{k in blk} s_i[m,k] x[k],   X[blk] = sum_{k in blk} x[k]
//
// HBM-bound by design: every plane word and scale is read once with 128-bit
// coalesced loads; the sign sums cost one LDS read and two VALU operations per
// 8 weights instead of one VALU operation per weight:
//
//  * A workgroup owns one column slice of 512 activations.  It first builds, in
//    LDS, one 256-entry fp32 table per 8 consecutive activations ("chunk"):
//    table[c][p] = sum_{b<8} (bit b of p ? +x : -x)[8c+b]  (the sign-sum lookup
//    idea of the LUT-GEMM kernel the paper cites, re-laid out for a conflict-free
//    access pattern): entry p of chunk c sits at byte p*256 + 4*c, so a chunk
//    lives in one LDS bank and the 64 chunks of the slice cover 64 dword columns.
//  * Each lane owns one (row, 128-column block, plane) at a time: 16 bytes of
//    sign bits = 16 table indices.  The packed blob stores a lane's 16 bytes
//    rotated by (row mod 16), so at lookup step j the 16 lanes that share a
//    block read 16 different chunks, and the four blocks of a wave are disjoint:
//    every ds_read_b32 of the wave is bank-conflict free.
//  * The LDS byte address (index*256 + 4*chunk) is assembled by one v_perm_b32
//    from a byte of the plane word and a byte of a per-lane constant.
//  * Lanes accumulate privately in fp32; the four block owners of a row are
//    summed once per 32-row tile with two lane-swap instructions
//    (v_permlane32_swap, v_permlane16_swap: vector ALU, no trip through LDS).
//  * Column slices are combined with ONE device-scope 64-bit integer atomic per
//    row and slice: the fp32 partial is converted to fixed point (2^-34 units,
//    54 bits, two's complement, wrapping) and added, together with an arrival
//    count in the low 10 bits, to the row's accumulator word in the workspace.
//    Integer addition commutes exactly, so the sum does not depend on arrival
//    order; the lane whose atomic returns the last arrival count owns the final
//    sum (returned value + own term), rounds it to binary16, stores y and
//    re-arms the word with zero.  No partial arrays, no fences, no second pass.
//  * Each wave double-buffers its tiles in registers: the loads of tile k+1 and the
//    split-K atomic of tile k-1 are in flight while tile k is computed; the value
//    an atomic returns is looked at one iteration after it was issued.
//  * The grid is exactly as large as the chip holds at once (two 64 KB-LDS
//    workgroups on each of the 256 CUs) whenever the problem is big enough, with
//    the column slices cut into unequal numbers of row parts to get there, so all
//    CUs carry the same load.  Workgroups have 8 waves (16 per CU) when every
//    wave still gets a tile, else 4.
//  * When a 128-column block holds several scaling groups (group 32 or 64) the
//    blob keeps each group in a fixed byte range of the lane's 16 bytes
//    (bcq_layout.h), so a lane sums its lookups per range and applies one alpha each.
#include <atomic>

#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct GemvParams {
    const uint8_t *blob;
    const uint16_t *x;
    uint16_t *y;
    unsigned long long *accum;  // [Mp] fixed-point row accumulators (value << 10 | arrivals)
    int M, N, Mp;
    int ntile, nslice;
    int parts, big_slices;  // slices [0, big_slices) have parts+1 workgroups, the others parts
    unsigned tile_bytes;
    int scale_lane_mask;  // 63: one scale record per lane; 15: one per row (group = N)
#ifdef BCQ_TRACE
    unsigned *trace;      // [workgroup][wave][kTraceSlots] time stamps (the tracing build only)
#endif
};

// Per-wave timeline for the tracing build (libbcq_trace.so, see trace_gemv.py): the 100 MHz real-time counter
// at fixed points, and the time spent in each part of the tile loop summed over the wave's tiles.  The normal
// build compiles none of this.
#ifdef BCQ_TRACE
#define BCQ_STAMP(i) (ts[i] = (unsigned)__builtin_amdgcn_s_memrealtime())
#define BCQ_PHASE(i)                                                      \
    do {                                                                  \
        asm volatile("" ::: "memory");                                    \
        const unsigned now_ = (unsigned)__builtin_amdgcn_s_memrealtime(); \
        ts[i] += now_ - tphase;                                           \
        tphase = now_;                                                    \
    } while (0)
#else
#define BCQ_STAMP(i) ((void)0)
#define BCQ_PHASE(i) ((void)0)
#endif


// One table lookup: byte `n` of plane word `w` is the index, byte `n` of `rv`
// is 4*chunk; the LDS byte address is index*256 + 4*chunk.
template <int n>
__device__ __forceinline__ float lookup(const float *lut, uint32_t w, uint32_t rv)
{
    constexpr uint32_t sel = 0x0c0c0000u | ((4u + n) << 8) | (uint32_t)n;
    uint32_t addr = __builtin_amdgcn_perm(w, rv, sel);
    return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lut) + addr);
}

// The 16 lookups of one (row, block, plane), summed per byte range: s[p] is the sign sum of
// the lane's bytes [16/SUB * p, 16/SUB * (p + 1)), i.e. of one scaling group.
template <int SUB>
__device__ __forceinline__ void sign_sums(const float *lut, const u32x4 &p, const uint32_t (&rv)[4], float (&s)[SUB])
{
    float d[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float a = lookup<0>(lut, p[v], rv[v]);
        a += lookup<1>(lut, p[v], rv[v]);
        a += lookup<2>(lut, p[v], rv[v]);
        a += lookup<3>(lut, p[v], rv[v]);
        d[v] = a;
    }
    if (SUB == 1) s[0] = (d[0] + d[1]) + (d[2] + d[3]);
    if (SUB == 2) { s[0] = d[0] + d[1]; s[SUB - 1] = d[2] + d[3]; }
    if (SUB == 4) {
#pragma unroll
        for (int v = 0; v < 4; ++v) s[v % SUB] = d[v];
    }
}

// Completes one row: `total` is the accumulator word after this slice's add.  The
// slice that arrives last converts the sum to binary16, stores it and zeroes the
// word for the next call.
__device__ __forceinline__ void complete_row(const GemvParams &p, int row, unsigned long long total)
{
    if (arrivals_of(total) == (unsigned)p.nslice) {
        if (row < p.M) p.y[row] = float_to_half_bits(decode_total(total));
        __hip_atomic_store(p.accum + row, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// EARLY = 1: no branch around the first loads (addresses are clamped instead), so that the wait in front of
// the table build can be for the activations alone and the tables are built while the first tile is still
// on its way.  Pays when a wave has a single tile (small layers: the kernel is one latency chain); with
// several tiles per wave it measured slower than waiting for both, so the launcher picks.
template <int Q, int Z, int NW, int SUB, int EARLY = 0>
__global__ __launch_bounds__(NW * 64) void bcq_gemv_kernel(GemvParams p)
{
    __shared__ float lut[256 * 64];  // 64 KB: entry idx of chunk c at lut[idx*64 + c]
#ifdef BCQ_TRACE
    unsigned ts[kTraceSlots] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, tphase = 0;
#endif
    BCQ_STAMP(0);  // wave started

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
    // Row tiles of this workgroup: an even split of the slice's tiles over its workgroups.  Inside the
    // workgroup wave w takes the tiles first + w, first + w + NW, ...: at any moment the workgroup
    // streams NW neighbouring tiles (one contiguous stretch of the blob), which the memory system serves
    // better than NW separate streams.
    const int g_begin = (int)(((long long)part * p.ntile) / parts);
    const int t_end = (int)(((long long)(part + 1) * p.ntile) / parts);
    const int t_begin = g_begin + wave < t_end ? g_begin + wave : t_end;
    const uint8_t *tile_ptr = p.blob + ((size_t)slice * p.ntile + t_begin) * p.tile_bytes;

    // Start the first tile's loads before building the tables.
    TileRegs<Q, Z, SUB> cur;
    const int col0 = slice * kTileCols + kChunkCols * lane;  // lane = chunk
    u32x4 xr = {0u, 0u, 0u, 0u};
    if (EARLY) {
        xr = *reinterpret_cast<const u32x4 *>(p.x + (col0 < p.N ? col0 : 0));
        // a wave without tiles reads the slice's last tile and drops it
        const int t_first = t_begin < p.ntile ? t_begin : p.ntile - 1;
        load_tile<Q, Z, SUB>(cur, p.blob + ((size_t)slice * p.ntile + t_first) * p.tile_bytes, lane,
                             lane & p.scale_lane_mask);
        if (col0 >= p.N) xr = u32x4{0u, 0u, 0u, 0u};
    } else {
        if (col0 < p.N) xr = *reinterpret_cast<const u32x4 *>(p.x + col0);
        if (t_begin < t_end) load_tile<Q, Z, SUB>(cur, tile_ptr, lane, lane & p.scale_lane_mask);
    }

    BCQ_STAMP(1);  // first loads issued
    // ---- sign-sum tables for the 512 activations of this slice ----------------
    {
        float xv[8];
        xv[0] = half_bits_to_float(xr.x & 0xffffu); xv[1] = half_bits_to_float(xr.x >> 16);
        xv[2] = half_bits_to_float(xr.y & 0xffffu); xv[3] = half_bits_to_float(xr.y >> 16);
        xv[4] = half_bits_to_float(xr.z & 0xffffu); xv[5] = half_bits_to_float(xr.z >> 16);
        xv[6] = half_bits_to_float(xr.w & 0xffffu); xv[7] = half_bits_to_float(xr.w >> 16);
#ifdef BCQ_TRACE
        asm volatile("" ::"v"(xv[0]), "v"(xv[7]));
#endif
        BCQ_STAMP(2);  // activations in registers (and, without EARLY, the first tile too)

        constexpr int IPW = 256 / NW;               // indices built by one wave
        constexpr int LB = (IPW == 64) ? 6 : (IPW == 32) ? 5 : (IPW == 128) ? 7 : 4;
        static_assert((1 << LB) == IPW, "NW must be 2, 4, 8 or 16");
        // bits >= LB of the index are fixed per wave
        float hi = 0.0f;
#pragma unroll
        for (int b = LB; b < 8; ++b) hi += ((wave >> (b - LB)) & 1) ? xv[b] : -xv[b];
        float lo[8];
#pragma unroll
        for (int a = 0; a < 8; ++a)
            lo[a] = ((a & 1) ? xv[0] : -xv[0]) + ((a & 2) ? xv[1] : -xv[1]) + ((a & 4) ? xv[2] : -xv[2]);
#pragma unroll
        for (int m = 0; m < IPW / 8; ++m) {
            float mid = hi;
#pragma unroll
            for (int b = 3; b < LB; ++b) mid += ((m >> (b - 3)) & 1) ? xv[b] : -xv[b];
#pragma unroll
            for (int a = 0; a < 8; ++a) lut[(wave * IPW + m * 8 + a) * 64 + lane] = lo[a] + mid;
        }
    }
    BCQ_STAMP(3);  // this wave's share of the tables written
    __syncthreads();
    BCQ_STAMP(4);  // tables complete

    // ---- per-lane constants ----------------------------------------------------
    const int r = lane & 15, h = lane >> 4;
    uint32_t rv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        uint32_t w = 0;
#pragma unroll
        for (int n = 0; n < 4; ++n) w |= (uint32_t)(4 * (16 * h + chunk_of_byte(4 * v + n, r, SUB))) << (8 * n);
        rv[v] = w;
    }
    float xsum[SUB];  // sums of the activations of this lane's block, per byte range (scaling group)
#pragma unroll
    for (int g = 0; g < SUB; ++g) {
        xsum[g] = 0.0f;
        if (Z) {
            const int c0 = (16 / SUB) * subgroup_of_range(g, r, SUB);
#pragma unroll
            for (int c = 0; c < 16 / SUB; ++c) xsum[g] += lut[255 * 64 + 16 * h + c0 + c];
        }
    }

    // ---- stream the row tiles ----------------------------------------------------
    // The split-K atomics are pipelined so that inside the loop no wave waits on a
    // round trip to memory that started less than one tile of work earlier.  With k
    // the tile computed in an iteration, the iteration
    //   (a) waits for all outstanding memory operations of the wave: the loads of
    //       tile k and the value returned by the atomic of tile k-2;
    //   (b) completes the rows of tile k-2 for which that value shows the last arrival;
    //   (c) issues the atomic of tile k-1, whose partial was kept in a register;
    //   (d) starts the loads of tile k+1;  (e) computes tile k.
    const bool split_k = p.nslice > 1;
    const bool reporter = (lane & 16) == 0;                      // lanes 0..15 and 32..47
    const int rep_row = (lane & 15) | ((lane >> 5) << 4);        // their row inside the tile
    int held_tile = -1;  // computed, partial still in `held`
    float held = 0.0f;
    int pend_tile = -1;  // atomic issued, result pending
    unsigned long long pend_old = 0, pend_mine = 0;

    for (int tile = t_begin; tile < t_end; tile += NW) {
#ifdef BCQ_TRACE
        tphase = (unsigned)__builtin_amdgcn_s_memrealtime();
#endif
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (a)
#ifdef BCQ_TRACE
        if (tile == t_begin) BCQ_STAMP(5);  // first tile in registers
        ts[15] += 1;
#endif
        BCQ_PHASE(8);  // waiting for the tile (and the atomic two tiles back)
        if (split_k && reporter) {
            if (pend_tile >= 0) complete_row(p, pend_tile * kTileRows + rep_row, pend_old + pend_mine);  // (b)
            pend_tile = held_tile;
            if (held_tile >= 0) {  // (c)
                pend_mine = encode_partial_f32(held);
                pend_old = __hip_atomic_fetch_add(p.accum + held_tile * kTileRows + rep_row, pend_mine,
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        BCQ_PHASE(9);  // completing rows, issuing the atomic
        TileRegs<Q, Z, SUB> nxt;
        tile_ptr += (size_t)NW * p.tile_bytes;
        if (tile + NW < t_end) load_tile<Q, Z, SUB>(nxt, tile_ptr, lane, lane & p.scale_lane_mask);  // (d)
        BCQ_PHASE(10);  // issuing the next tile's loads (stalls here when the memory pipeline is full)

        float acc[2];  // (e)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                float ss[SUB];
                sign_sums<SUB>(lut, cur.planes[t][i], rv, ss);
#pragma unroll
                for (int g = 0; g < SUB; ++g) a = fmaf(scale_of<Q, Z, SUB>(cur, t, g, i), ss[g], a);
            }
            if (Z) {
#pragma unroll
                for (int g = 0; g < SUB; ++g) a = fmaf(scale_of<Q, Z, SUB>(cur, t, g, Q), xsum[g], a);
            }
            acc[t] = a;
        }
        // the four block owners (lanes r, r+16, r+32, r+48) of each row summed: rows 0..15 of the tile
        // end up in the lanes 0..15, rows 16..31 in the lanes 32..47 (the reporters)
#ifdef BCQ_TRACE
        asm volatile("" ::"v"(acc[0]), "v"(acc[1]));
#endif
        BCQ_PHASE(11);  // table look-ups and scaling
        const float out = sum_block_owners(acc[0], acc[1]);
        if (split_k) {
            held = out;
            held_tile = tile;
        } else {
            const int row = tile * kTileRows + rep_row;
            if (reporter && row < p.M) p.y[row] = float_to_half_bits(out);
        }
#ifdef BCQ_TRACE
        asm volatile("" ::"v"(out));
#endif
        BCQ_PHASE(12);  // cross-lane sum
        if (tile + NW < t_end) cur = nxt;
    }
    BCQ_STAMP(6);  // tile loop left

    if (split_k && reporter) {  // drain: two tiles may still be in the pipeline
        if (held_tile >= 0) {
            const unsigned long long mine = encode_partial_f32(held);
            const unsigned long long old = __hip_atomic_fetch_add(p.accum + held_tile * kTileRows + rep_row, mine,
                                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (pend_tile >= 0) complete_row(p, pend_tile * kTileRows + rep_row, pend_old + pend_mine);
            complete_row(p, held_tile * kTileRows + rep_row, old + mine);
        } else if (pend_tile >= 0) {
            complete_row(p, pend_tile * kTileRows + rep_row, pend_old + pend_mine);
        }
    }
#ifdef BCQ_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    BCQ_STAMP(7);  // last atomic returned, last store acknowledged
    if (p.trace && lane == 0) {
        unsigned *dst = p.trace + ((size_t)blockIdx.x * NW + wave) * kTraceSlots;
#pragma unroll
        for (int i = 0; i < kTraceSlots; ++i) dst[i] = ts[i];
    }
#endif
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
// Workgroups of the GEMV the current device holds at once: every instantiation uses 64 KB of LDS and at most 128
// registers, so the occupancy of one of them, asked from the runtime once per device, stands for all (two per
// compute unit on gfx950: 512 on an MI355X).
int resident_gemv_groups()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 2 * 256;
    int groups = cached[dev].load(std::memory_order_relaxed);
    if (groups == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bcq_gemv_kernel<3, 0, 8, 1>, 8 * 64, 0) != hipSuccess ||
            per_cu < 1)
            per_cu = 2;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        groups = per_cu * cus;
        cached[dev].store(groups, std::memory_order_relaxed);
    }
    return groups;
}

int auto_workgroups(const Geom &g, int waves_per_group)
{
    // All workgroups resident at once and doing equal work; at least one tile per wave.
    long long tiles = (long long)g.nslice * g.ntile;
    long long groups = (tiles + waves_per_group - 1) / waves_per_group;
    const int resident = resident_gemv_groups();
    if (groups > resident) groups = resident;
    if (groups < 1) groups = 1;
    return (int)groups;
}

template <int Q, int Z, int NW, int SUB, int EARLY = 0>
static hipError_t launch_one(const GemvParams &p, int groups, hipStream_t stream)
{
    hipLaunchKernelGGL((bcq_gemv_kernel<Q, Z, NW, SUB, EARLY>), dim3((unsigned)groups), dim3(NW * 64), 0,
                       stream, p);
    return hipGetLastError();
}

template <int Q, int Z>
static hipError_t launch_qz(const GemvParams &p, int waves, int sub, int groups, bool early, hipStream_t stream)
{
    if (sub == 2) return launch_one<Q, Z, 4, 2>(p, groups, stream);
    if (sub == 4) return launch_one<Q, Z, 4, 4>(p, groups, stream);
    if (early) return waves == 8 ? launch_one<Q, Z, 8, 1, 1>(p, groups, stream) : launch_one<Q, Z, 4, 1, 1>(p, groups, stream);
    return waves == 8 ? launch_one<Q, Z, 8, 1>(p, groups, stream) : launch_one<Q, Z, 4, 1>(p, groups, stream);
}

// The launch shape: workgroups, waves per workgroup, start-up order.
void gemv_launch_shape(const Geom &g, const GemvTuning &t, int *groups_out, int *waves_out, bool *early_out)
{
    // measured: from about four tiles per resident workgroup on, eight waves win (7168 x 7168: 392 workgroups of
    // 8 waves with one tile each 7.4 us, 512 of 4 waves 8.0 us; 1024 x 8192: 4 waves 4.2 us, 8 waves 4.7 us);
    // the variants with several scaling groups per block exist with 4 waves only
    const long long tiles = (long long)g.nslice * g.ntile;
    const int want = t.waves ? t.waves : (tiles >= 4LL * resident_gemv_groups() ? 8 : 4);
    const int nw = (want == 8 && g.sub == 1) ? 8 : 4;
    int groups = t.workgroups > 0 ? t.workgroups : auto_workgroups(g, nw);
    // at least one workgroup per slice, at most one per row tile of a slice
    if (groups < g.nslice) groups = g.nslice;
    if ((long long)groups > tiles) groups = (int)tiles;
    // one tile per wave at most: the early table build pays (measured: 7168 x 7168 8.0 -> 7.4 us, 8192 x 8192
    // 8.55 -> 8.3 us, 1024 x 8192 5.0 -> 4.2 us; with more tiles per wave it loses 1.5-2 us on the large layers)
    *early_out = t.early ? t.early == 1 : tiles <= (long long)groups * nw;
    *groups_out = groups;
    *waves_out = nw;
}

hipError_t launch_gemv(const Geom &g, const void *packed, const uint16_t *x, uint16_t *y,
                       void *workspace, const GemvTuning &t, hipStream_t stream)
{
    int groups, nw;
    bool early;
    gemv_launch_shape(g, t, &groups, &nw, &early);
    GemvParams p;
    p.parts = groups / g.nslice;
    p.big_slices = groups % g.nslice;
    p.blob = static_cast<const uint8_t *>(packed);
    p.x = x;
    p.y = y;
    p.accum = static_cast<unsigned long long *>(workspace);
    p.M = g.M; p.N = g.N; p.Mp = g.Mp;
    p.ntile = g.ntile; p.nslice = g.nslice;
    p.tile_bytes = g.tile_bytes;
    p.scale_lane_mask = g.scale_lanes - 1;
#ifdef BCQ_TRACE
    p.trace = static_cast<unsigned *>(t.trace);
#endif
    const int key = g.q * 2 + g.z;
    switch (key) {
        case 2: return launch_qz<1, 0>(p, nw, g.sub, groups, early, stream);
        case 3: return launch_qz<1, 1>(p, nw, g.sub, groups, early, stream);
        case 4: return launch_qz<2, 0>(p, nw, g.sub, groups, early, stream);
        case 5: return launch_qz<2, 1>(p, nw, g.sub, groups, early, stream);
        case 6: return launch_qz<3, 0>(p, nw, g.sub, groups, early, stream);
        case 7: return launch_qz<3, 1>(p, nw, g.sub, groups, early, stream);
        case 8: return launch_qz<4, 0>(p, nw, g.sub, groups, early, stream);
        case 9: return launch_qz<4, 1>(p, nw, g.sub, groups, early, stream);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------
// streaming-read probe: same load width and a similar launch shape, no arithmetic
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4 *__restrict__ buf, size_t n16,
                                                         uint32_t *__restrict__ sink)
{
    // each workgroup reads one contiguous span; each wave keeps 4 KB (4 loads of 16 B per lane) in flight
    constexpr int U = 4;
    size_t per_block = (n16 + gridDim.x - 1) / gridDim.x;
    per_block = (per_block + 256 * U - 1) / (256 * U) * (256 * U);
    const size_t begin = (size_t)blockIdx.x * per_block;
    const size_t end = begin + per_block < n16 ? begin + per_block : n16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t acc = 0;
    for (size_t i = begin + wave * (64 * U) + lane; i < end; i += 256 * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t idx = i + u * 64;
            v[u] = idx < end ? __builtin_nontemporal_load(buf + idx) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    acc ^= __shfl_xor(acc, 32, 64);
    acc ^= __shfl_xor(acc, 16, 64);
    acc ^= __shfl_xor(acc, 8, 64);
    acc ^= __shfl_xor(acc, 4, 64);
    acc ^= __shfl_xor(acc, 2, 64);
    acc ^= __shfl_xor(acc, 1, 64);
    __shared__ uint32_t part[4];
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

hipError_t launch_read_probe(const void *buf, size_t bytes, void *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(read_probe_kernel, dim3(kProbeBlocks), dim3(256), 0, stream,
                       static_cast<const u32x4 *>(buf), bytes / 16, static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace bcq
