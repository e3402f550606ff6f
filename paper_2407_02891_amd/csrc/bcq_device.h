// Device-side helpers shared by the GEMV and skinny kernels (not public).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bcq {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 128-bit load

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float v)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));  // round to nearest even
}

// One tile's share of a lane.  SUB = scaling groups per 128-column block (1, 2 or 4).
template <int Q, int Z, int SUB = 1>
struct TileRegs {
    u32x4 planes[2][Q];
    uint32_t scales[(Q + Z) * SUB];  // binary16 pairs: [t][range][c] flattened, 2*SUB*(Q+Z) halves
};

// `scale_lane` = index of the lane's scale record: the lane itself, or lane mod 16 when the
// scales are stored once per row (see bcq_layout.h).
template <int Q, int Z, int SUB>
__device__ __forceinline__ void load_tile(TileRegs<Q, Z, SUB> &r, const uint8_t *tile, int lane, int scale_lane)
{
    const u32x4 *pp = reinterpret_cast<const u32x4 *>(tile) + lane;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < Q; ++i) r.planes[t][i] = __builtin_nontemporal_load(pp + (t * Q + i) * 64);
    const uint32_t *sp = reinterpret_cast<const uint32_t *>(tile + 2u * Q * 1024u) + scale_lane * ((Q + Z) * SUB);
#pragma unroll
    for (int c = 0; c < (Q + Z) * SUB; ++c) r.scales[c] = __builtin_nontemporal_load(sp + c);
}

// dword 3 of a raw buffer descriptor (no swizzle, no stride, 32-bit data format)
constexpr int kRawBufferFlags = 0x00020000;

// The same tile through a buffer descriptor whose range is the tile (or empty): a load outside
// the range returns zeros without touching memory.  Lets a loop request "the next tile, if any"
// without a branch, so that the compiler can count the outstanding loads instead of draining them.
template <int Q, int Z, int SUB>
__device__ __forceinline__ void load_tile_buf(TileRegs<Q, Z, SUB> &r, __amdgpu_buffer_rsrc_t rsrc, int lane,
                                              int scale_lane)
{
    constexpr int kNonTemporal = 2;
    const uint32_t po = 16u * lane;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < Q; ++i)
            r.planes[t][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, po + (t * Q + i) * 1024u, 0, kNonTemporal);
    const uint32_t so = 2u * Q * 1024u + 4u * (Q + Z) * SUB * scale_lane;
#pragma unroll
    for (int c = 0; c < (Q + Z) * SUB; ++c)
        r.scales[c] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, so + 4u * c, 0, kNonTemporal);
}

// One piece of the same requests: piece k < 2 Q is sign plane k (row half k div Q, plane k mod Q), piece
// 2 Q the scale record.  For kernels that spread the requests over their compute steps.
template <int Q, int Z, int SUB>
__device__ __forceinline__ void load_tile_piece(TileRegs<Q, Z, SUB> &r, __amdgpu_buffer_rsrc_t rsrc, int lane,
                                                int scale_lane, int piece)
{
    constexpr int kNonTemporal = 2;
    if (piece < 2 * Q) {
        r.planes[piece / Q][piece % Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, 16u * lane + piece * 1024u, 0, kNonTemporal);
    } else {
        const uint32_t so = 2u * Q * 1024u + 4u * (Q + Z) * SUB * scale_lane;
#pragma unroll
        for (int c = 0; c < (Q + Z) * SUB; ++c)
            r.scales[c] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, so + 4u * c, 0, kNonTemporal);
    }
}

// binary16 bits of scale c (alpha_0..alpha_{Q-1}, then the offset) of row half t, byte range `range`
template <int Q, int Z, int SUB>
__device__ __forceinline__ uint32_t scale_bits_of(const TileRegs<Q, Z, SUB> &r, int t, int range, int c)
{
    const int e = (t * SUB + range) * (Q + Z) + c;  // half index
    const uint32_t pair = r.scales[e >> 1];
    return (e & 1) ? (pair >> 16) : (pair & 0xffffu);
}

template <int Q, int Z, int SUB>
__device__ __forceinline__ float scale_of(const TileRegs<Q, Z, SUB> &r, int t, int range, int c)
{
    return half_bits_to_float(scale_bits_of<Q, Z, SUB>(r, t, range, c));
}

// Split-K accumulator word: bits 63..10 = sum of the slices' partials in units of
// 2^-34 (two's complement, wraps modulo 2^54), bits 9..0 = number of slices that
// have arrived.  A slice adds (fixed << 10) + 1.
constexpr int kCountBits = 10;
constexpr double kFixedScale = 17179869184.0;  // 2^34

__device__ __forceinline__ unsigned long long encode_partial(float v)
{
    // keep the conversion in range; magnitudes this large cannot end in a finite binary16
    v = fminf(fmaxf(v, -536870848.0f), 536870848.0f);  // |v| < 2^29
    long long fixed = __double2ll_rn(static_cast<double>(v) * kFixedScale);  // exact product
    return (static_cast<unsigned long long>(fixed) << kCountBits) + 1ull;
}

// The same word without binary64 instructions (about half the vector-ALU work; used by the GEMV, whose
// loop is short enough for it to matter).
__device__ __forceinline__ unsigned long long encode_partial_f32(float v)
{
    // keep the conversion in range; magnitudes this large cannot end in a finite binary16
    v = fminf(fmaxf(v, -536870848.0f), 536870848.0f);  // |v| < 2^29
    // round(v * 2^34) as a 64-bit two's complement integer, in binary32 steps that are all exact: the
    // product is a power-of-two scaling; rintf leaves an integer m of at most 24 significant bits below
    // 2^63; its magnitude splits as hi * 2^32 + lo with 0 <= lo < 2^32, both representable (when hi > 0,
    // lo is a multiple of ulp(m) >= 2^9).  The sign is applied to the 64-bit integer afterwards (a
    // negative value cannot be split the same way: -5 = -1 * 2^32 + 4294967291 needs 32 bits).
    const float m = fabsf(rintf(v * 17179869184.0f));
    const float hi = floorf(m * 2.3283064365386963e-10f);
    const float lo = fmaf(-hi, 4294967296.0f, m);
    const unsigned long long mag = (static_cast<unsigned long long>(static_cast<unsigned>(hi)) << 32) |
                                   static_cast<unsigned long long>(static_cast<unsigned>(lo));
    // two's complement negation where v is negative, without a lane mask: (mag ^ s) - s, s = 0 or all ones
    const unsigned long long sgn = static_cast<unsigned long long>(static_cast<long long>(static_cast<int>(__float_as_uint(v)) >> 31));
    const unsigned long long fixed = (mag ^ sgn) - sgn;
    return (fixed << kCountBits) + 1ull;
}

// Value of a completed accumulator word (arrival count dropped).
__device__ __forceinline__ float decode_total(unsigned long long total)
{
    const long long fixed = static_cast<long long>(total) >> kCountBits;
    return static_cast<float>(static_cast<double>(fixed) * (1.0 / kFixedScale));
}

// Sum over the four lanes l, l^16, l^32, l^48 (the owners of the four 128-column blocks of a row) of `a0`
// in the lanes 0..15 (and 16..31) and of `a1` in the lanes 32..47 (and 48..63), with two lane-swap
// instructions on the vector ALU instead of four trips through the LDS crossbar.
__device__ __forceinline__ float sum_block_owners(float a0, float a1)
{
    // upper half of a0 <-> lower half of a1: lanes 0..31 then hold a0's two row pairs, lanes 32..63 a1's
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(a0), __float_as_uint(a1), false, false);
    const unsigned h0 = h[0], h1 = h[1];  // (element reads first: a bit cast straight from h[1] reads h[0])
    const float s = __uint_as_float(h0) + __uint_as_float(h1);
    // odd 16-lane rows of one copy <-> even rows of the other: every row of 16 lanes then sees both halves
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return __uint_as_float(r0) + __uint_as_float(r1);
}

// Work split of the kernels that walk along K (bcq_skinny.hip, bcq_lut4.hip): `units` work items are cut into one
// contiguous range per workgroup, of floor or ceil(units / workgroups) items.  Two ways to place the longer ranges:
//
// FRONT (kernels that run one workgroup per compute unit): the first `rem` = units mod workgroups of the workgroups
// take `base` + 1 = floor(units / workgroups) + 1 items, the others `base`.  The hardware starts the workgroups in
// order, so the longer ranges begin up to 0.7 us before the last ones (measured: 1 us per launch on a layer with
// 1.5 items per workgroup).  The host passes base and rem.
//
// Otherwise the longer ranges are spread evenly over the workgroup numbers (range w = [floor(w units / groups),
// floor((w + 1) units / groups))): with two workgroups per compute unit, numbers w and w + groups / 2 typically
// share one, and the front placement would give some compute units two long ranges (4.6 us on a 45 us launch).  The
// kernel of bcq_lut4.hip keeps the even spread too: its long ranges placed at the front lie next to each other in
// memory and cost 2 to 3 us on layers with five or six items per workgroup.
//
// First item of workgroup w, and the workgroup that owns item u.
template <bool FRONT>
__device__ __forceinline__ int first_unit(int w, int units, int groups, int base, int rem)
{
    if (FRONT) return w * base + (w < rem ? w : rem);
    return (int)(((long long)w * units) / groups);
}

template <bool FRONT>
__device__ __forceinline__ int owner_of_unit(int u, int units, int groups, int base, int rem)
{
    if (FRONT) {
        const int cut = rem * (base + 1);  // items of the longer ranges (base = 0 only if every item is below `cut`)
        const long long n = u < cut ? u : u - cut, d = u < cut ? base + 1 : base;
        return (u < cut ? 0 : rem) + (int)(n / d);
    }
    return (int)((((long long)u + 1) * groups - 1) / units);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned arrivals_of(unsigned long long total)
{
    return static_cast<unsigned>(total) & ((1u << kCountBits) - 1u);
}

}  // namespace bcq
