// Skinny binary-coding GEMM for gfx950: Y[j][m] = sum_k W_q[m][k] X[j][k] for 2 <= batch <= 64
// (paper Eq. 11 applied to a few activation vectors at once), reading the packed weights ONCE.
//
// With several activation vectors the work per weight bit grows with the batch while the
// bytes do not, so the path stops being HBM-bound and the sign-sum tables of the batch-1
// kernel (one table set per activation vector) no longer fit in LDS.  Here every sign becomes
// a binary16 operand of the matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulate); the cost
// is the same for every batch up to 16; wider batches (up to 64) reuse the expanded operands for
// every group of 16 columns.
//
// Common skeleton (bcq_skinny_kernel<Q, Z, SUB, VER, LDS_STEPS, NB, NW>):
//  * Same packed blob as the GEMV (bcq_layout.h).  A work unit is (tile group, column slice): the
//    NW (4 or 8) waves of a workgroup take the NW row tiles of the group and share an LDS copy of the
//    slice of X (pitch 1040 B: conflict-free ds_read_b128; double-buffered, one barrier per unit).
//    The units, ordered tile group first, are cut into equal contiguous ranges, one per workgroup,
//    with as many workgroups as the chip holds at once: every workgroup does the same number of
//    units (+-1) whatever the shape.  (Cutting finer, in 128-column blocks, was measured and lost: a
//    unit done in part still pays its tile, its X slice and its barrier.)  When a range leaves a tile group the accumulators are
//    flushed; the workgroups that share a tile group are combined with the same fixed-point 64-bit
//    atomics as in the GEMV (the expected number of arrivals follows from the ranges).
//  * Tile and X loads go through buffer descriptors (empty / out of range when there is no next
//    unit) so that the loop has no branch around them and the compiler counts outstanding loads.
//  * Before the flush the 32 x 16 result block of a wave is turned through LDS so that a store or
//    atomic instruction covers whole 64-byte lines.
//
// Two ways to form the A operand:
//  VER 1 (any group size): lane l = 16h + r holds the 128 sign bits of (row r, block h, plane i)
//    -- exactly the A-operand ownership of the MFMA (row = l mod 16, k-octet = l div 16) -- so one
//    MFMA step mixes four blocks, i.e. four scaling groups, and alpha is folded into A: one byte
//    of signs -> 8 values +-alpha with 1 v_perm_b32 + 4 x (shift, and-or).  The offset term is one
//    more MFMA per chunk with A = (z, ..., z).  Bound: vector ALU.
//  VER 2 (one scaling group per 128-column block): the four lanes that hold the four blocks of
//    one row exchange dwords (4 x 4 transpose, v_permlane16_swap / v_permlane32_swap), after
//    which lane (h, r) holds, for EVERY block B of row r, the chunks 4h..4h+3, and one MFMA step
//    contracts 32 columns of a single block.  A is then just +-1.0, independent of the row: it
//    comes from a 256-entry table in LDS (one ds_read_b128 per 8 signs; 8 interleaved copies so
//    that neighbouring lanes read different banks); LDS_STEPS of the 4 steps of a block use the
//    table, the others expand in registers.  The products of one block are collected in a
//    temporary accumulator and scaled by alpha (fp32) when the block is done; the scales are
//    fetched into the accumulator's row layout with ds_bpermute.  The offset term uses A = all
//    ones: the block's column sums of X, scaled by z.  Bound: LDS read bandwidth.
//  In both, the pairing inside an octet (elements 2d, 2d+1 <-> columns d, d+4) is arbitrary as
//  long as A and B agree; X is stored in LDS in that order.
#include <atomic>

#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct SkinnyParams {
    const uint8_t *blob;
    const uint16_t *X;
    uint16_t *Y;
    unsigned long long *accum;  // [batch][Mp]
    int M, N, Mp, batch, ldx, ldy;
    int ntile, nslice, ntg;  // ntg = ceil(ntile / 4) tile groups (the four row tiles of a workgroup)
    int units;               // ntg * nslice work units, cut into one contiguous range per workgroup:
    int unit_base, unit_rem; // units div / mod the number of workgroups (first_unit, owner_of_unit in bcq_device.h)
    unsigned tile_bytes;
    int scale_lane_mask;     // 63: one scale record per lane; 15: one per row (group = N)
#ifdef BCQ_TRACE
    unsigned *trace;         // [workgroup][wave][kTraceSlots] time stamps (the tracing build only)
    int trace_groups;        // workgroups the buffer has room for
#endif
};

// Per-wave timeline for the tracing build (libbcq_trace.so, see trace_gemv.py): the 100 MHz real-time
// counter at fixed points and the time spent in each part of a work unit, summed over the wave's units.
// The normal build compiles none of this.
#ifdef BCQ_TRACE
#define BCQ_SK_NOW() ((unsigned)__builtin_amdgcn_s_memrealtime())
#define BCQ_SK_STAMP(i) (ts[i] = BCQ_SK_NOW())
#define BCQ_SK_PHASE(i)                 \
    do {                                \
        const unsigned now_ = BCQ_SK_NOW(); \
        ts[i] += now_ - last;           \
        last = now_;                    \
    } while (0)
#else
#define BCQ_SK_STAMP(i) ((void)0)
#define BCQ_SK_PHASE(i) ((void)0)
#endif

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Staged X in LDS: one row of 64 chunks (16 B each) per batch column, rows `pitch` bytes apart.  A
// ds_read_b128 is served 16 lanes at a time -- lanes {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19,
// 28-31} and the same plus 32 -- and such a group runs at full rate when its 16 addresses fall in 16
// different 16-byte columns of the 256-byte bank row (measured on gfx950; 64 banks of 4 bytes).
//  VER 1 reads (row r, chunk 16 h + k): pitch 1040 puts row r in column r + k.
//  VER 2 reads (row r, chunk 16 B + 4 h + s) for one (B, s) at a time: the chunks of a block are stored
//    in the order 4 s + h and the pitch is 1056, which puts lane (h, r) in column 2 r + h + 4 s.
template <int VER> constexpr int kXPitch = VER == 2 ? 1056 : 1040;
template <int VER> constexpr int kXBuf = 16 * kXPitch<VER>;

// Loads (into registers) this thread's share of the X slice (16 NB batch rows): 4 NB chunks of 8 activations.  X is read
// through a buffer descriptor covering its batch rows; chunks that do not exist (batch column or
// column out of range, or no such slice: `wanted` false) are given an out-of-range offset and
// come back as zeros, so the loads are unconditional.
template <int NB, int NT>
__device__ __forceinline__ void x_slice_load(const SkinnyParams &p, __amdgpu_buffer_rsrc_t xrsrc, int slice, bool wanted,
                                             int tid, u32x4 (&xr)[1024 * NB / NT])
{
#pragma unroll
    for (int k = 0; k < 1024 * NB / NT; ++k) {
        const int idx = tid + NT * k, chunk = idx & 63, c = idx >> 6;
        const int col = slice * kTileCols + kChunkCols * chunk;
        const bool ok = wanted && c < p.batch && col < p.N;
        const uint32_t off = ok ? 2u * ((uint32_t)c * (uint32_t)p.ldx + (uint32_t)col) : 0xfffffff0u;
        xr[k] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0);
    }
}

// Descriptor of the activations: rows 0 .. batch-1 of X (batch * ldx binary16 values).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t x_descriptor(const SkinnyParams &p)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.X), 0, (int)(2u * (uint32_t)p.batch * (uint32_t)p.ldx),
                                             kRawBufferFlags);
}

// Descriptor of one tile, or an empty one.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_descriptor(const uint8_t *tile, unsigned tile_bytes, bool wanted)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(tile), 0, wanted ? (int)tile_bytes : 0, kRawBufferFlags);
}

// Stores them to LDS, elements reordered to (0,4,1,5,2,6,3,7) within a chunk.
template <int NB, int NT, int VER>
__device__ __forceinline__ void x_slice_store(uint8_t *xs, int tid, const u32x4 (&xr)[1024 * NB / NT])
{
#pragma unroll
    for (int k = 0; k < 1024 * NB / NT; ++k) {
        const int idx = tid + NT * k, chunk = idx & 63, c = idx >> 6;
        const u32x4 v = xr[k];
        u32x4 o;
        o.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);  // (x0, x4)
        o.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);  // (x1, x5)
        o.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);  // (x2, x6)
        o.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);  // (x3, x7)
        // VER 2: chunk 4 h + s of a block sits at position 4 s + h
        const int pos = VER == 2 ? ((chunk & 48) | ((chunk & 3) << 2) | ((chunk >> 2) & 3)) : chunk;
        // VER 2: batch column h + 4 j of a group of 16 goes to row 4 h + j, so that the lanes 16 h + r of the (transposed)
        // MFMA result hold the columns h, h + 4, h + 8, h + 12: a flush instruction then covers four neighbouring columns
        const int row = VER == 2 ? ((c & ~15) | ((c & 3) << 2) | ((c >> 2) & 3)) : c;
        *reinterpret_cast<u32x4 *>(xs + row * kXPitch<VER> + pos * 16) = o;
    }
}

// Undo the per-row byte permutation of the blob (chunk_of_byte): on return byte s of the
// 128-bit value is chunk s.
template <int SUB>
__device__ __forceinline__ void unrotate(u32x4 &w, int r)
{
    if (SUB == 1) {
        // chunk = (byte + r) mod 16: rotate the 128-bit ring left by r bytes, i.e. right by k = (16 - r) mod 16:
        // byte j of the result is byte j + k of w.  Dword step first (two rounds of selects), then one
        // v_alignbyte_b32 per dword for the k mod 4 bytes that cross dwords.
        const int k = (16 - r) & 15;
        const bool s1 = k & 4, s2 = k & 8;
        const uint32_t b = k & 3;
        uint32_t t0 = w.x, t1 = w.y, t2 = w.z, t3 = w.w;
        const uint32_t u0 = s1 ? t1 : t0, u1 = s1 ? t2 : t1, u2 = s1 ? t3 : t2, u3 = s1 ? t0 : t3;
        t0 = s2 ? u2 : u0; t1 = s2 ? u3 : u1; t2 = s2 ? u0 : u2; t3 = s2 ? u1 : u3;
        w.x = __builtin_amdgcn_alignbyte(t1, t0, b);
        w.y = __builtin_amdgcn_alignbyte(t2, t1, b);
        w.z = __builtin_amdgcn_alignbyte(t3, t2, b);
        w.w = __builtin_amdgcn_alignbyte(t0, t3, b);
    } else if (SUB == 2) {  // rotate each 64-bit half left by r mod 8 bytes, swap the halves if r >= 8
        unsigned long long lo = ((unsigned long long)w.y << 32) | w.x, hi = ((unsigned long long)w.w << 32) | w.z;
        lo = __builtin_rotateleft64(lo, 8 * (r & 7));
        hi = __builtin_rotateleft64(hi, 8 * (r & 7));
        const unsigned long long a = (r & 8) ? hi : lo, b = (r & 8) ? lo : hi;
        w.x = (uint32_t)a; w.y = (uint32_t)(a >> 32); w.z = (uint32_t)b; w.w = (uint32_t)(b >> 32);
    } else {  // rotate each dword left by r mod 4 bytes, dword d goes to d xor (r div 4)
        const unsigned sh = 8 * (r & 3);
        uint32_t t0 = __builtin_rotateleft32(w.x, sh), t1 = __builtin_rotateleft32(w.y, sh);
        uint32_t t2 = __builtin_rotateleft32(w.z, sh), t3 = __builtin_rotateleft32(w.w, sh);
        // masked exchanges (written without selects so that they stay in registers)
        const uint32_t m4 = (r & 4) ? 0xffffffffu : 0u, m8 = (r & 8) ? 0xffffffffu : 0u;
        uint32_t d01 = (t0 ^ t1) & m4, d23 = (t2 ^ t3) & m4;
        t0 ^= d01; t1 ^= d01; t2 ^= d23; t3 ^= d23;
        uint32_t d02 = (t0 ^ t2) & m8, d13 = (t1 ^ t3) & m8;
        t0 ^= d02; t2 ^= d02; t1 ^= d13; t3 ^= d13;
        w.x = t0; w.y = t1; w.z = t2; w.w = t3;
    }
}

// Eight binary16 values (bit ? +|a| : -|a|), after the caller has pre-inverted the word for
// non-negative alpha: pair d of the result takes its signs from bits d and d+4 of byte n of w.
template <int n>
__device__ __forceinline__ f16x8 expand_byte(uint32_t w, uint32_t w_shr4, uint32_t abs_pair)
{
    // r = (byte n of w) << 8 | (byte n of w >> 4) << 24
    constexpr uint32_t sel = ((uint32_t)n << 24) | (0x0cu << 16) | ((4u + n) << 8) | 0x0cu;
    const uint32_t r = __builtin_amdgcn_perm(w, w_shr4, sel);
    u32x4 a;
    a.x = ((r << 7) & 0x80008000u) | abs_pair;
    a.y = ((r << 6) & 0x80008000u) | abs_pair;
    a.z = ((r << 5) & 0x80008000u) | abs_pair;
    a.w = ((r << 4) & 0x80008000u) | abs_pair;
    return __builtin_bit_cast(f16x8, a);
}

// Scale c of row half t for scaling sub-group g of the block (chunk order).  The lane stores its
// scales per byte range; the range that holds sub-group g depends on the lane, so every range
// is read and one is kept (no dynamic register index).
template <int Q, int Z, int SUB>
__device__ __forceinline__ uint32_t scale_bits(const TileRegs<Q, Z, SUB> &t, int th, int g, int r, int c)
{
    const int range = subgroup_of_range(g, r, SUB);  // an involution: range <-> sub-group
    if (SUB == 1) return scale_bits_of<Q, Z, SUB>(t, th, 0, c);
    uint32_t v = 0;  // and-or with masks rather than selects: stays in registers
#pragma unroll
    for (int k = 0; k < SUB; ++k) v |= scale_bits_of<Q, Z, SUB>(t, th, k, c) & ((range == k) ? 0xffffffffu : 0u);
    return v;
}

// Adds the wave's partial results to the outputs.  On entry acc[t][i] = partial of row
// 32*tile + 16*t + 4*h + i for batch column r (the MFMA accumulator layout, lane = 16h + r).  The
// 32 x 16 block is first turned through LDS (`stage`, private to the wave, kStageFloats floats) so
// that lanes 0..31 and 32..63 each hold 32 consecutive rows of one batch column: a store or atomic
// instruction then covers whole 64-byte lines of Y / of the accumulator words instead of
// scattered 8-byte pieces.  `col0` = first batch column of the block; `arrivals` = number of workgroups that contribute to this tile group:
// with one the values are stored directly; otherwise they are combined with the fixed-point
// split-K atomics (see bcq_device.h).
constexpr int kStagePitch = 33;
constexpr int kStageFloats = 17 * kStagePitch + 15;  // 576

template <int ROUND, bool TRANSPOSED>
__device__ __forceinline__ void skinny_store(const SkinnyParams &p, const f32x4 (&acc)[2], int tile, int lane,
                                             float *stage, int arrivals, int col0)
{
    const int r = lane & 15, h = lane >> 4;
    // acc[t][i] is (row 16t + 4h + i, column r) of the tile, or with TRANSPOSED (row 16t + r, column h + 4i)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (TRANSPOSED) stage[(h + 4 * i) * kStagePitch + 16 * t + r] = acc[t][i];
            else stage[r * kStagePitch + 16 * t + 4 * h + i] = acc[t][i];
        }
    // same wave: its LDS operations complete in order, no barrier needed
    const int row = tile * kTileRows + (lane & 31), half = lane >> 5;
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = stage[(2 * k + half) * kStagePitch + (lane & 31)];
    if (arrivals == 1) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int col = col0 + 2 * k + half;
            if (col < p.batch && row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(v[k]);
        }
        return;
    }
    // ROUND atomics in flight at once (8: one round trip to the L2 per flush; 4 where registers are short)
#pragma unroll
    for (int k0 = 0; k0 < 8; k0 += ROUND) {
        unsigned long long mine[ROUND], old[ROUND];
#pragma unroll
        for (int k = 0; k < ROUND; ++k) {
            const int col = col0 + 2 * (k0 + k) + half;
            mine[k] = encode_partial(v[k0 + k]);
            old[k] = 0;
            if (col < p.batch)
                old[k] = __hip_atomic_fetch_add(p.accum + (size_t)col * p.Mp + row, mine[k], __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int k = 0; k < ROUND; ++k) {
            const int col = col0 + 2 * (k0 + k) + half;
            const unsigned long long total = old[k] + mine[k];
            if (col < p.batch && arrivals_of(total) == (unsigned)arrivals) {
                if (row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(decode_total(total));
                __hip_atomic_store(p.accum + (size_t)col * p.Mp + row, 0ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// The same for accumulators held transposed (the table kernel): acc[t][j] = (batch column col0 + h + 4j, row 16t + r)
// of the tile, lane 16h + r.  No turn through LDS: an instruction's lanes cover 16 consecutive rows of four neighbouring
// columns, and with few columns the instructions for j beyond them have no active lane.
template <int ROUND>
__device__ __forceinline__ void skinny_store_transposed(const SkinnyParams &p, const f32x4 (&acc)[2], int tile, int lane,
                                                        int arrivals, int col0)
{
    const int r = lane & 15, h = lane >> 4;
    if (arrivals == 1) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int col = col0 + h + 4 * (k & 3), row = tile * kTileRows + 16 * (k >> 2) + r;
            if (col < p.batch && row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(acc[k >> 2][k & 3]);
        }
        return;
    }
#pragma unroll
    for (int k0 = 0; k0 < 8; k0 += ROUND) {
        unsigned long long mine[ROUND], old[ROUND];
#pragma unroll
        for (int k = 0; k < ROUND; ++k) {
            const int col = col0 + h + 4 * ((k0 + k) & 3), row = tile * kTileRows + 16 * ((k0 + k) >> 2) + r;
            mine[k] = encode_partial(acc[(k0 + k) >> 2][(k0 + k) & 3]);
            old[k] = 0;
            if (col < p.batch)
                old[k] = __hip_atomic_fetch_add(p.accum + (size_t)col * p.Mp + row, mine[k], __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int k = 0; k < ROUND; ++k) {
            const int col = col0 + h + 4 * ((k0 + k) & 3), row = tile * kTileRows + 16 * ((k0 + k) >> 2) + r;
            const unsigned long long total = old[k] + mine[k];
            if (col < p.batch && arrivals_of(total) == (unsigned)arrivals) {
                if (row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(decode_total(total));
                __hip_atomic_store(p.accum + (size_t)col * p.Mp + row, 0ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// VER 1: one tile and slice, alpha folded into A
// ---------------------------------------------------------------------------------
template <int Q, int Z, int SUB, int NB>
__device__ __forceinline__ void compute_folded(TileRegs<Q, Z, SUB> &cur, const uint8_t *xs_buf, int r, int h,
                                               f32x4 (&acc)[NB][2])
{
    // per (row half, plane): un-rotate, fold the sign of alpha into the bits, |alpha| pair
    uint32_t abs_pair[2][Q][SUB];
    uint32_t z_pair[2][SUB];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            u32x4 w = cur.planes[t][i];
            unrotate<SUB>(w, r);
            uint32_t flip[SUB];
#pragma unroll
            for (int g = 0; g < SUB; ++g) {
                const uint32_t ab = scale_bits<Q, Z, SUB>(cur, t, g, r, i);
                flip[g] = (ab & 0x8000u) ? 0u : 0xffffffffu;  // bit 1 <-> +1
                const uint32_t mag = ab & 0x7fffu;
                abs_pair[t][i][g] = mag | (mag << 16);
            }
            // dword d of the un-permuted value belongs to sub-group d * SUB / 4
            w.x ^= flip[0];
            w.y ^= flip[SUB == 4 ? 1 : 0];
            w.z ^= flip[SUB == 4 ? 2 : SUB - 1];
            w.w ^= flip[SUB - 1];
            cur.planes[t][i] = w;
        }
        if (Z) {
#pragma unroll
            for (int g = 0; g < SUB; ++g) {
                const uint32_t zb = scale_bits<Q, Z, SUB>(cur, t, g, r, Q);
                z_pair[t][g] = zb | (zb << 16);
            }
        }
    }
    const uint8_t *xb = xs_buf + r * kXPitch<1> + h * 256;
#pragma unroll
    for (int dq = 0; dq < 4; ++dq) {
        constexpr int per = 4 / SUB;  // dwords (of 4 chunks) per scaling sub-group
        const int g = dq / per;
        uint32_t w[2][Q], w4[2][Q];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                w[t][i] = cur.planes[t][i][dq];
                w4[t][i] = w[t][i] >> 4;
            }
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            // the expanded operands of a step serve every group of 16 batch columns
            f16x8 bx[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                bx[nb] = *reinterpret_cast<const f16x8 *>(xb + nb * kXBuf<1> + (4 * dq + n) * 16);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    f16x8 a;
                    if (n == 0) a = expand_byte<0>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                    if (n == 1) a = expand_byte<1>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                    if (n == 2) a = expand_byte<2>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                    if (n == 3) a = expand_byte<3>(w[t][i], w4[t][i], abs_pair[t][i][g]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bx[nb], acc[nb][t], 0, 0, 0);
                }
                if (Z) {
                    const u32x4 zz = {z_pair[t][g], z_pair[t][g], z_pair[t][g], z_pair[t][g]};
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, zz), bx[nb], acc[nb][t],
                                                                            0, 0, 0);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// VER 2: lane transpose, +-1.0 operands from the LDS table, alpha applied to the accumulators
// ---------------------------------------------------------------------------------
// Sign table: entry b holds 8 binary16 values, pair d = (bit d, bit d + 4) of b, +1.0 for a set bit
// (the element order the staged X uses); copy c of entry b sits at (TC b + c) * 16 and lane l reads copy
// l mod TC.  With TC = 16 copies (64 KB) the 16 lanes that a ds_read_b128 serves together always read 16
// different bank columns whatever their bytes are; with 8 copies (32 KB) two of them share a column and
// collide unless their bytes are equal, which costs the table reads about half their rate.
template <int TC> constexpr int kTabBytes = 256 * TC * 16;

template <int NT, int TC>
__device__ __forceinline__ void build_sign_table(uint8_t *tab, int tid)
{
#pragma unroll
    for (int k = 0; k < 256 * TC / NT; ++k) {
        const int idx = tid + NT * k, b = idx / TC;
        u32x4 e;
#pragma unroll
        for (int d = 0; d < 4; ++d)
            e[d] = (((b >> d) & 1) ? 0x3c00u : 0xbc00u) | ((((b >> (d + 4)) & 1) ? 0x3c00u : 0xbc00u) << 16);
        *reinterpret_cast<u32x4 *>(tab + idx * 16) = e;
    }
}

// `issue(g)` is called after the MFMAs of step g = 4 B + s (0..15): the kernel uses it to request the next
// unit's tile and X slice a piece at a time.  Requested all at once at the top of a unit, the 8 waves of a
// workgroup queue up behind each other in the CU's vector-memory pipeline (measured: up to 1.4 us per unit
// for the wave that comes last, and everyone waits for it at the barrier).
template <int Q, int Z, int LDS_STEPS, int NB, int TC, class Issue>
__device__ __forceinline__ void compute_table(const TileRegs<Q, Z, 1> &cur, const uint8_t *xs_buf, const uint8_t *tab,
                                              uint32_t copy_bits, int r, int h, f32x4 (&acc)[NB][2], unsigned &t_operands,
                                              Issue issue)
{
    // chunk order, then the 4 x 4 dword transpose across the lanes r, r+16, r+32, r+48:
    // wb[t][i][B] = chunks 4h .. 4h+3 of (row 16t + r, block B, plane i)
    uint32_t wb[2][Q][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            u32x4 w = cur.planes[t][i];
            unrotate<1>(w, r);
            const auto e01 = __builtin_amdgcn_permlane16_swap(w.x, w.y, false, false);
            const auto e23 = __builtin_amdgcn_permlane16_swap(w.z, w.w, false, false);
            const auto f02 = __builtin_amdgcn_permlane32_swap(e01[0], e23[0], false, false);
            const auto f13 = __builtin_amdgcn_permlane32_swap(e01[1], e23[1], false, false);
            wb[t][i][0] = f02[0]; wb[t][i][1] = f13[0]; wb[t][i][2] = f02[1]; wb[t][i][3] = f13[1];
        }
#ifdef BCQ_TRACE
    asm volatile("" : "+v"(wb[1][Q - 1][3]));  // the tile has arrived and is transposed
    t_operands = BCQ_SK_NOW();
#else
    (void)t_operands;
#endif
    // The products are formed transposed (batch columns as the rows of the MFMA result): lane 16 h + r then holds four
    // batch columns (h + 4 j, see x_slice_store) of weight row r, whose scales for block B sit in lane 16 B + r.  One copy of every
    // lane group's scale record in every lane group: three lane-swap instructions per dword, once per unit.
    uint32_t sc[4][Q + Z];
#pragma unroll
    for (int e = 0; e < Q + Z; ++e) {
        const uint32_t v = cur.scales[e];
        const auto lo_hi = __builtin_amdgcn_permlane32_swap(v, v, false, false);  // lane groups (0,1,0,1), (2,3,2,3)
        const unsigned lo = lo_hi[0], hi = lo_hi[1];
        const auto g01 = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);  // (0,0,0,0), (1,1,1,1)
        const auto g23 = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);  // (2,2,2,2), (3,3,3,3)
        sc[0][e] = g01[0]; sc[1][e] = g01[1]; sc[2][e] = g23[0]; sc[3][e] = g23[1];
    }
    // batch column 16 nb + r of the staged X sits in row 16 nb + r of the buffer
    const uint8_t *xb = xs_buf + r * kXPitch<2> + h * 16;
    const u32x4 ones = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
#pragma unroll
    for (int B = 0; B < 4; ++B) {
        f32x4 C[NB][2][Q];  // first written by the MFMAs of step 0, whose addend is the constant zero
        f32x4 Cz[NB];
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        // The +-1.0 operands of a step serve every group of 16 batch columns.  With four groups a
        // wave runs alone on its SIMD (registers, LDS), so nothing else hides the LDS latency: the
        // operands of step s+1 are requested before the MFMAs of step s are issued (with one or two
        // groups two waves share a SIMD and the extra registers of that pipelining would cost one).
        constexpr bool kPipelined = NB == 4;
        auto fetch = [&](int s, f16x8 (&a)[2][Q], f16x8 (&bx)[NB]) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    const uint32_t w = wb[t][i][B];
                    if (s < LDS_STEPS) {
                        if constexpr (TC == 16) {
                            // 256 bytes per entry: byte s of w becomes byte 1 of the offset, the lane's copy
                            // (bits 4..7) byte 0 -- one v_perm_b32 per look-up
                            const uint32_t off = __builtin_amdgcn_perm(w, copy_bits, 0x0c0c0400u | ((uint32_t)s << 8));
                            a[t][i] = *reinterpret_cast<const f16x8 *>(tab + off);
                        } else {
                            const uint32_t byte = (w >> (8 * s)) & 0xffu;
                            a[t][i] = *reinterpret_cast<const f16x8 *>(tab + copy_bits + byte * (16 * TC));
                        }
                    } else {
                        const uint32_t wn = ~w, wn4 = wn >> 4;
                        if (s == 0) a[t][i] = expand_byte<0>(wn, wn4, 0x3c003c00u);
                        if (s == 1) a[t][i] = expand_byte<1>(wn, wn4, 0x3c003c00u);
                        if (s == 2) a[t][i] = expand_byte<2>(wn, wn4, 0x3c003c00u);
                        if (s == 3) a[t][i] = expand_byte<3>(wn, wn4, 0x3c003c00u);
                    }
                }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                bx[nb] = *reinterpret_cast<const f16x8 *>(xb + nb * kXBuf<2> + (16 * B + 4 * s) * 16);
        };
        f16x8 abuf[2][2][Q], bbuf[2][NB];
        fetch(0, abuf[0], bbuf[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int cb = s & 1;
            if (kPipelined) {
                if (s + 1 < 4) fetch(s + 1, abuf[cb ^ 1], bbuf[cb ^ 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < Q; ++i)
                        C[nb][t][i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bbuf[cb][nb], abuf[cb][t][i],
                                                                             s == 0 ? zero : C[nb][t][i], 0, 0, 0);
                if (Z)
                    Cz[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bbuf[cb][nb], __builtin_bit_cast(f16x8, ones),
                                                                    s == 0 ? zero : Cz[nb], 0, 0, 0);
            }
            if (kPipelined) __builtin_amdgcn_sched_barrier(0);
            else if (s + 1 < 4) fetch(s + 1, abuf[cb ^ 1], bbuf[cb ^ 1]);  // left to the compiler's schedule
            issue(4 * B + s);
        }
        // acc[nb][t][j] (batch column 16 nb + h + 4j, row 16t + r) += alpha_i(row, block B) * C[nb][t][i][j]  (+ z * column sums)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < Q + Z; ++c) {
                const int e = t * (Q + Z) + c;  // half index in the scale record
                const uint32_t pair = sc[B][e >> 1];
                const float v = half_bits_to_float((e & 1) ? (pair >> 16) : (pair & 0xffffu));
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb][t][j] = fmaf(v, c < Q ? C[nb][t][c < Q ? c : 0][j] : Cz[nb][j], acc[nb][t][j]);
            }
    }
}

// ---------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------
// NB = groups of 16 batch columns (1, 2 or 4; with VER 1 or VER 2).  With one group the
// X slice is double-buffered in LDS; with more, the staged slice (16.6 KB per group) is single-
// buffered: the next slice waits in registers and replaces it between two barriers.
template <int Q, int Z, int SUB, int VER, int LDS_STEPS, int NB, int NW>
__global__ __launch_bounds__(64 * NW) void bcq_skinny_kernel(SkinnyParams p)
{
    constexpr int NT = 64 * NW;
    static_assert(VER == 1 || SUB == 1, "the table kernel needs one scaling group per block");
    // Eight waves: registers allow one workgroup per CU (two waves per SIMD from q = 2 on), which leaves
    // room for 16 table copies and two X buffers.
    constexpr bool kDouble = NB == 1;
    constexpr int TC = NW == 8 ? 16 : 8;
    constexpr int kBuf = NB * kXBuf<VER>;
    __shared__ __attribute__((aligned(16))) uint8_t xs[(kDouble ? 2 : 1) * kBuf];
    __shared__ __attribute__((aligned(16))) uint8_t tab[VER == 2 ? kTabBytes<TC> : 16];
    __shared__ float stage[VER == 2 && NB < 4 ? 1 : NW * kStageFloats];  // (the direct flush does not turn its results through LDS)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: tile pointers stay in SGPRs
    const int r = lane & 15, h = lane >> 4;
#ifdef BCQ_TRACE
    unsigned ts[kTraceSlots] = {};
    unsigned last = 0;
#endif
    BCQ_SK_STAMP(0);  // wave started
    constexpr bool kFront = NW == 8;  // eight waves: one workgroup per compute unit (LDS, registers)
    const int groups = gridDim.x;
    const int u_begin = first_unit<kFront>(blockIdx.x, p.units, groups, p.unit_base, p.unit_rem);
    const int u_end = first_unit<kFront>(blockIdx.x + 1, p.units, groups, p.unit_base, p.unit_rem);
    if (u_begin >= u_end) return;  // uniform for the workgroup, before any barrier

    int tg = u_begin / p.nslice, slice = u_begin - tg * p.nslice;
    int tile = NW * tg + wave;
    bool active = tile < p.ntile;

    const __amdgpu_buffer_rsrc_t xrsrc = x_descriptor(p);
    TileRegs<Q, Z, SUB> cur;
    load_tile_buf<Q, Z, SUB>(
        cur, tile_descriptor(p.blob + ((size_t)slice * p.ntile + (active ? tile : 0)) * p.tile_bytes, p.tile_bytes, active),
        lane, lane & p.scale_lane_mask);
    {
        u32x4 xr[1024 * NB / NT];
        x_slice_load<NB, NT>(p, xrsrc, slice, true, tid, xr);
        x_slice_store<NB, NT, VER>(xs, tid, xr);
    }
    if (VER == 2) build_sign_table<NT, TC>(tab, tid);
    __syncthreads();
    const uint32_t copy_bits = (lane & (TC - 1)) * 16;  // byte offset of this lane's copy inside a table entry
    BCQ_SK_STAMP(1);  // first X slice staged, sign table built

    int buf = 0;
    int u = u_begin;
    while (u < u_end) {
        // one segment: the units of this workgroup that belong to tile group `tg`
        const int seg_end = min(u_end, (tg + 1) * p.nslice);
        const int seg_tile = tile;
        const bool seg_active = active;
        // number of workgroups that contribute to this tile group; worked out here and parked in a vector register,
        // because at the flush the kernels with four column groups have no scalar register to spare
        int seg_arrivals = owner_of_unit<kFront>((tg + 1) * p.nslice - 1, p.units, groups, p.unit_base, p.unit_rem) -
                           owner_of_unit<kFront>(tg * p.nslice, p.units, groups, p.unit_base, p.unit_rem) + 1;
        asm volatile("" : "+v"(seg_arrivals));
        f32x4 acc[NB][2];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb][0] = acc[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (; u < seg_end; ++u) {
            // the next unit of this workgroup, if any (it may be the first of the next segment)
#ifdef BCQ_TRACE
            last = BCQ_SK_NOW();
            ts[15] += 1;
#endif
            const bool more = u + 1 < u_end;
            int n_slice = slice + 1, n_tg = tg;
            if (n_slice == p.nslice) { n_slice = 0; n_tg = tg + 1; }
            const int n_tile = NW * n_tg + wave;
            const bool n_active = more && n_tile < p.ntile;
            // unconditional requests for it (empty descriptor / out-of-range offsets when there is
            // none): they stay in flight while this unit is computed
            TileRegs<Q, Z, SUB> nxt;
            u32x4 xr[1024 * NB / NT];
            const __amdgpu_buffer_rsrc_t n_rsrc = tile_descriptor(
                p.blob + ((size_t)n_slice * p.ntile + (n_active ? n_tile : 0)) * p.tile_bytes, p.tile_bytes, n_active);
            // The table kernel spreads these requests over its MFMA steps: the X slice after step 0, two
            // sign planes after each of the next Q steps, then the scales; the rest of the unit covers
            // their latency.
            constexpr bool kSpread = VER == 2;
            auto issue = [&](int g) {
                if (g == 0) x_slice_load<NB, NT>(p, xrsrc, n_slice, more, tid, xr);
                if (g >= 1 && g <= Q) {
                    load_tile_piece<Q, Z, SUB>(nxt, n_rsrc, lane, lane & p.scale_lane_mask, 2 * (g - 1));
                    load_tile_piece<Q, Z, SUB>(nxt, n_rsrc, lane, lane & p.scale_lane_mask, 2 * (g - 1) + 1);
                }
                if (g == Q + 1) load_tile_piece<Q, Z, SUB>(nxt, n_rsrc, lane, lane & p.scale_lane_mask, 2 * Q);
            };
            if (!kSpread || !active) {
                load_tile_buf<Q, Z, SUB>(nxt, n_rsrc, lane, lane & p.scale_lane_mask);
                x_slice_load<NB, NT>(p, xrsrc, n_slice, more, tid, xr);
            }
            BCQ_SK_PHASE(12);  // top of the unit: addresses of the next one (and its requests, unless spread)

            if (active) {
                if constexpr (VER == 1) compute_folded<Q, Z, SUB, NB>(cur, xs + buf * kBuf, r, h, acc);
                else {
                    unsigned t_operands = 0;
                    compute_table<Q, Z, LDS_STEPS, NB, TC>(cur, xs + buf * kBuf, tab, copy_bits, r, h, acc, t_operands, issue);
#ifdef BCQ_TRACE
                    ts[8] += t_operands - last;  // next unit's loads issued, this tile arrived, un-rotated and transposed
                    last = t_operands;
                    asm volatile("" : "+v"(acc[0][0][0]), "+v"(acc[0][1][3]));
#endif
                }
            }
            BCQ_SK_PHASE(9);  // the MFMA steps of the unit
            if (!kDouble) __syncthreads();  // everyone done reading the slice that is about to be replaced
            if (more) {
                x_slice_store<NB, NT, VER>(xs + (kDouble ? (buf ^ 1) * kBuf : 0), tid, xr);
                cur = nxt;
            }
            tg = n_tg; slice = n_slice; tile = n_tile; active = n_active;
            if (kDouble) buf ^= 1;
            BCQ_SK_PHASE(10);  // next X slice (waited for and) stored to LDS
            __syncthreads();  // next X slice written (double-buffered: and everyone done with the current one)
            BCQ_SK_PHASE(11);  // waiting for the other waves at the barrier
        }
        BCQ_SK_STAMP(2);  // (last) segment's units done
        // this workgroup is done with the tile group: flush (the next segment's first loads are in flight)
        if (seg_active) {
            const int arrivals = __builtin_amdgcn_readfirstlane(seg_arrivals);
            // (the lane index is passed through an empty asm so that the per-lane address arithmetic of
            // the flush is not hoisted out of this loop into registers that stay live during the units)
            int flush_lane = lane;
            asm volatile("" : "+v"(flush_lane));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                // (four column groups: the kernel has no scalar registers left for the direct form's column tests)
                if constexpr (VER == 2 && NB < 4)
                    skinny_store_transposed<NB == 1 ? 8 : 4>(p, acc[nb], seg_tile, flush_lane, arrivals, 16 * nb);
                else
                    skinny_store<NB == 1 ? 8 : 4, VER == 2>(p, acc[nb], seg_tile, flush_lane, stage + wave * kStageFloats, arrivals, 16 * nb);
            }
        }
    }
#ifdef BCQ_TRACE
    __builtin_amdgcn_s_waitcnt(0);
    BCQ_SK_STAMP(3);  // last flush done
    if (p.trace && lane == 0 && (int)blockIdx.x < p.trace_groups) {
        unsigned *dst = p.trace + ((size_t)blockIdx.x * 8 + wave) * kTraceSlots;  // 8 records per workgroup
        for (int i = 0; i < kTraceSlots; ++i) dst[i] = ts[i];
    }
#endif
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
// Number of workgroups of a kernel the current device holds at once (asked once per kernel).
template <int Q, int Z, int SUB, int VER, int LDS_STEPS, int NB, int NW>
static int resident_groups()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];  // per device (zero-initialised)
    int dev = 0;
    const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices;
    int groups = known ? cached[dev].load(std::memory_order_relaxed) : 0;
    if (groups == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bcq_skinny_kernel<Q, Z, SUB, VER, LDS_STEPS, NB, NW>, 64 * NW,
                                                         0) != hipSuccess ||
            per_cu < 1)
            per_cu = 1;
        if (!known || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        groups = per_cu * cus;
        if (known) cached[dev].store(groups, std::memory_order_relaxed);
    }
    return groups;
}

// Grid size: `parts` > 0: that many workgroups per tile group (a K split); `parts` < 0: -parts
// workgroups; 0: as many workgroups as are resident.
template <int Q, int Z, int SUB, int VER, int LDS_STEPS, int NB, int NW = 4>
static hipError_t launch_skinny_one(SkinnyParams p, int parts, bool single_slice, hipStream_t stream)
{
    p.ntg = (p.ntile + NW - 1) / NW;  // the NW waves of a workgroup take the NW row tiles of a tile group
    const long long units = (long long)p.ntg * p.nslice;
    if (units > 0x7fffffffLL) return hipErrorInvalidValue;
    p.units = (int)units;
    long long groups = parts > 0 ? (long long)parts * p.ntg
                                 : parts < 0 ? -(long long)parts : resident_groups<Q, Z, SUB, VER, LDS_STEPS, NB, NW>();
    if (groups > p.units) groups = p.units;
    if (single_slice) groups = p.ntg;  // no workspace: one unit per tile group, nothing to combine
    if (groups < 1) groups = 1;
    p.unit_base = (int)(p.units / groups);
    p.unit_rem = (int)(p.units % groups);
    hipLaunchKernelGGL((bcq_skinny_kernel<Q, Z, SUB, VER, LDS_STEPS, NB, NW>), dim3((unsigned)groups), dim3(64 * NW), 0,
                       stream, p);
    return hipGetLastError();
}

// One launch for up to 16 NB batch columns; p.X / p.Y / p.accum / p.batch describe exactly those.
template <int Q, int Z>
static hipError_t launch_skinny_qz(const SkinnyParams &p, int nb, int parts, bool single_slice, int sub, int version,
                                   int lds_steps, int waves, hipStream_t stream)
{
    if (sub == 2) return launch_skinny_one<Q, Z, 2, 1, 0, 1>(p, parts, single_slice, stream);
    if (sub == 4) return launch_skinny_one<Q, Z, 4, 1, 0, 1>(p, parts, single_slice, stream);
    // Which kernel (measured on 7168 x 28672, q = 3, eager launches): up to 16 columns the table kernel (42 against
    // 55 us for the kernel that folds alpha into A); 17 to 32 columns the table kernel with two column groups and
    // eight waves where it exists (60 against 70 us), else the alpha-folding kernel; beyond 32 columns the alpha-folding
    // kernel (118 against 126 us at 64): its expansion is shared by the column groups like the table kernel's, it
    // needs no per-block accumulators, and the table kernel with four column groups has four waves and 8 table
    // copies only.
    const long long tiles = (long long)p.ntile * p.nslice;
    const bool table2 = nb == 2 && Q <= 3 && (waves == 8 || (waves == 0 && tiles >= 2048));
    if (version == 1 || (version == 0 && nb > 1 && !table2)) {
        if (nb == 4) return launch_skinny_one<Q, Z, 1, 1, 0, 4>(p, parts, single_slice, stream);
        // 32 columns: eight waves per workgroup from 4096 tiles on (63 against 73 us on 7168 x 28672)
        if (nb == 2 && (waves == 8 || (waves == 0 && tiles >= 4096)))
            return launch_skinny_one<Q, Z, 1, 1, 0, 2, 8>(p, parts, single_slice, stream);
        if (nb == 2) return launch_skinny_one<Q, Z, 1, 1, 0, 2>(p, parts, single_slice, stream);
        return launch_skinny_one<Q, Z, 1, 1, 0, 1>(p, parts, single_slice, stream);
    }
    if constexpr (Q <= 3) {  // with four planes, four column groups do not fit the table kernel's register budget
        if (nb == 4) return launch_skinny_one<Q, Z, 1, 2, 4, 4>(p, parts, single_slice, stream);
    }
    if constexpr (Q <= 3) {  // four planes exceed 256 registers with two column groups and eight waves
        if (table2) return launch_skinny_one<Q, Z, 1, 2, 4, 2, 8>(p, parts, single_slice, stream);
    }
    if (nb == 2) return launch_skinny_one<Q, Z, 1, 2, 4, 2>(p, parts, single_slice, stream);
    // all four MFMA steps of a block from the LDS table measured fastest; 3 (one step expanded in
    // registers) is kept as the alternative for tuning runs
    // Eight waves per workgroup (eight row tiles share one staged slice of X; one workgroup per CU, which
    // leaves LDS for 16 conflict-free table copies) win from about 2000 tiles on (measured at batch 4 / 16,
    // eager launches: 7168 x 28672 39.4 / 41.4 against 46.0 / 48.1 us, 36864 x 9216 56 / 60 against 67 / 70,
    // 9216 x 9216 25.1 / 27.2 against 27.5 / 29.2, 7168 x 7168 20.7 / 23.4 against 22.4 / 24.2,
    // 12288 x 4096 20.9 / 23.1 against 22.3 / 24.0; 4096 x 4096 and below: four waves by 0.4 to 1.5 us).
    const bool eight = waves == 8 || (waves == 0 && tiles >= 2048);
    if (eight && lds_steps != 3) return launch_skinny_one<Q, Z, 1, 2, 4, 1, 8>(p, parts, single_slice, stream);
    return lds_steps == 3 ? launch_skinny_one<Q, Z, 1, 2, 3, 1>(p, parts, single_slice, stream)
                          : launch_skinny_one<Q, Z, 1, 2, 4, 1>(p, parts, single_slice, stream);
}

hipError_t launch_skinny(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy,
                         int batch, void *workspace, const GemvTuning &tuning, hipStream_t stream)
{
    // Up to four vectors, three or four planes, large layers: sign-sum tables with the four sums side by side
    // (bcq_lut4.hip).  Measured against the matrix-core kernel, q = 3, batch 2 / 4: 7168 x 28672 31.2 / 32.8 against
    // 32.4 / 31.8 us, 28672 x 8192 33.2 / 35.5 against 37.4 / 33.7, 36864 x 9216 42.6 / 44.6 against 49.3 / 46.0,
    // 9216 x 36864 41.9 / 44.5 against 49.4 / 45.9: with two vectors it wins from about 12000 tiles on, with three or
    // four only on the largest layers; it loses on smaller ones (9216 x 9216: 21.3 / 24.1 against 18.3 / 18.2) and
    // with one or two planes (its table builds and barriers do not shrink with q).
    const long long all_tiles = (long long)g.ntile * g.nslice;
    // Two vectors: the GEMV's decomposition with both vectors' sign sums in one table entry (bcq_gemv2.hip).  Measured
    // against the best of the kernels below, q = 3: 7168 x 28672 23.6 against 32.4 us, 28672 x 7168 22.5 / 32.1,
    // 9216 x 36864 36.3 / 49.4, 9216 x 9216 12.7 / 17.4, 7168 x 7168 10.7 / 13.1 (q = 2, 7168 x 28672: 18.0 / 22.8); it
    // loses where a compute unit gets less than a round of tiles (4096 x 4096 9.1 / 8.6, 1024 x 8192 8.8 / 7.9).
    if (gemv2_applies(g, batch, workspace) &&
        (tuning.skinny_version == 5 || (tuning.skinny_version == 0 && all_tiles >= 2048)))
        return launch_gemv2(g, packed, X, ldx, Y, ldy, workspace, tuning, stream);
    // (versions 5 and 6 only switch the two-vector kernel on and off: automatic choice among the others)
    const int version = tuning.skinny_version >= 5 ? 0 : tuning.skinny_version;
    if (lut4_applies(g, batch, workspace) &&
        (version == 3 ||
         (version == 0 && g.q >= 3 && all_tiles >= (batch == 2 ? 12288 : 18432))))
        return launch_lut4(g, packed, X, ldx, Y, ldy, batch, workspace, tuning, stream);
    SkinnyParams p;
    p.blob = static_cast<const uint8_t *>(packed);
    p.M = g.M; p.N = g.N; p.Mp = g.Mp; p.ldx = ldx; p.ldy = ldy;
    p.ntile = g.ntile; p.nslice = g.nslice; p.ntg = 0; p.units = 0; p.unit_base = 0; p.unit_rem = 0;  // set per kernel (waves per workgroup)
    p.tile_bytes = g.tile_bytes;
    p.scale_lane_mask = g.scale_lanes - 1;
#ifdef BCQ_TRACE
    p.trace = static_cast<unsigned *>(tuning.trace);
    p.trace_groups = tuning.trace_groups;
#endif
    // forced grid sizes (tuning runs, tests): a K split per tile group, or a plain number of workgroups
    const int parts = tuning.skinny_parts > 0 ? tuning.skinny_parts : -tuning.workgroups;
    const bool single = workspace == nullptr;  // only reachable for a single column slice
    const int sub = g.sub, ver = version, steps = tuning.skinny_lds_steps;
    // Up to 64 batch columns in one pass over the weights (the expanded operands are shared by the
    // groups of 16 columns); with several scaling groups per block one pass per 16 columns.
    const bool wide_ok = sub == 1;
    const int widest = (g.q <= 3 || ver != 2) ? 64 : 32;
    const int cols_per_launch = wide_ok ? (batch > 32 ? widest : batch > 16 ? 32 : 16) : 16;
    for (int col0 = 0; col0 < batch; col0 += cols_per_launch) {
        const int cols = batch - col0 < cols_per_launch ? batch - col0 : cols_per_launch;
        p.X = X + (size_t)col0 * ldx;
        p.Y = Y + (size_t)col0 * ldy;
        p.accum = static_cast<unsigned long long *>(workspace) + (workspace ? (size_t)col0 * g.Mp : 0);
        p.batch = cols;
        const int nb = cols > 32 ? 4 : cols > 16 ? 2 : 1;
        hipError_t e = hipErrorInvalidValue;
        switch (g.q * 2 + g.z) {
            case 2: e = launch_skinny_qz<1, 0>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 3: e = launch_skinny_qz<1, 1>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 4: e = launch_skinny_qz<2, 0>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 5: e = launch_skinny_qz<2, 1>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 6: e = launch_skinny_qz<3, 0>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 7: e = launch_skinny_qz<3, 1>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 8: e = launch_skinny_qz<4, 0>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
            case 9: e = launch_skinny_qz<4, 1>(p, nb, parts, single, sub, ver, steps, tuning.waves, stream); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace bcq
