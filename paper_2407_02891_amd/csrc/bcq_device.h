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

// Value of a completed accumulator word (arrival count dropped).
__device__ __forceinline__ float decode_total(unsigned long long total)
{
    const long long fixed = static_cast<long long>(total) >> kCountBits;
    return static_cast<float>(static_cast<double>(fixed) * (1.0 / kFixedScale));
}

__device__ __forceinline__ unsigned arrivals_of(unsigned long long total)
{
    return static_cast<unsigned>(total) & ((1u << kCountBits) - 1u);
}

}  // namespace bcq
