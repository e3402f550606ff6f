// Skinny binary-coding GEMM for gfx950: Y[j][m] = sum_k W_q[m][k] X[j][k] for 2 <= batch <= 16
// (paper Eq. 11 applied to a few activation vectors at once), reading the packed weights ONCE.
//
// With several activation vectors the work per weight bit grows with the batch while the
// bytes do not, so the path stops being HBM-bound and the sign-sum tables of the batch-1
// kernel (one table set per activation vector) no longer fit in LDS.  Here the planes are
// instead expanded in registers to binary16 values +-alpha and contracted with the
// activations on the matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulate): the cost is
// the same for every batch up to 16.
//
//  * Same packed blob as the GEMV (bcq_layout.h).  A wave owns one 32-row tile and walks over
//    the column slices of its K-part; lane l = 16h + r holds, per row half t and plane i, the
//    128 sign bits of (row 16t + r, 128-column block h) -- exactly the A-operand ownership of
//    the MFMA (row = l mod 16, k-octet = l div 16).  The GEMV's per-row byte rotation is undone
//    once per 128 bits (a dword rotate and a funnel shift).
//  * One MFMA step contracts chunk s (8 columns) of all four blocks: A = 8 binary16 values
//    (sign ? +alpha : -alpha) built from one byte of sign bits with 1 v_perm_b32 + 4 x
//    (shift, and-or); B = the 8 activations of that chunk for batch column l mod 16, one
//    ds_read_b128 from a staged copy of X (pitch 1040 B: conflict-free).  alpha is folded into A
//    because the four k-octets of one MFMA belong to four different scaling groups.
//    The pairing inside an octet (elements 2d, 2d+1 <-> columns d, d+4) is arbitrary as long
//    as A and B agree; X is stored in LDS in that order.
//  * The offset term of Eq. 11 is one more MFMA per chunk with A = (z, z, ..., z).
//  * The four waves of a workgroup work on four adjacent row tiles and share the staged X
//    slice (double-buffered, one barrier per slice).
//  * K is split into `parts` so that ~2000 waves exist; the parts are combined with the same
//    fixed-point 64-bit atomics as in the GEMV (one per output element and part).
#include "bcq_internal.h"
#include "bcq_device.h"

namespace bcq {

struct SkinnyParams {
    const uint8_t *blob;
    const uint16_t *X;
    uint16_t *Y;
    unsigned long long *accum;  // [batch][Mp]
    int M, N, Mp, batch, ldx, ldy;
    int ntile, nslice, ntg, parts;  // ntg = ceil(ntile / 4) tile groups
    unsigned tile_bytes;
};

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kXPitchBytes = 1040;  // 64 chunks x 16 B + 16 B: batch rows land in different banks
constexpr int kXBufBytes = 16 * kXPitchBytes;

// Loads (into registers) this thread's share of the X slice: 4 chunks of 8 activations.
__device__ __forceinline__ void x_slice_load(const SkinnyParams &p, int slice, int tid, u32x4 (&xr)[4])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int idx = tid + 256 * k, chunk = idx & 63, c = idx >> 6;
        const int col = slice * kTileCols + kChunkCols * chunk;
        xr[k] = u32x4{0u, 0u, 0u, 0u};
        if (c < p.batch && col < p.N)
            xr[k] = *reinterpret_cast<const u32x4 *>(p.X + (size_t)c * p.ldx + col);
    }
}

// Stores them to LDS, elements reordered to (0,4,1,5,2,6,3,7) within a chunk.
__device__ __forceinline__ void x_slice_store(uint8_t *xs, int tid, const u32x4 (&xr)[4])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int idx = tid + 256 * k, chunk = idx & 63, c = idx >> 6;
        const u32x4 v = xr[k];
        u32x4 o;
        o.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);  // (x0, x4)
        o.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);  // (x1, x5)
        o.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);  // (x2, x6)
        o.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);  // (x3, x7)
        *reinterpret_cast<u32x4 *>(xs + c * kXPitchBytes + chunk * 16) = o;
    }
}

// Undo the per-row byte permutation of the blob (chunk_of_byte): on return byte s of the
// 128-bit value is chunk s.
template <int SUB>
__device__ __forceinline__ void unrotate(u32x4 &w, int r)
{
    if (SUB == 1) {  // chunk = (byte + r) mod 16: rotate the 128-bit ring left by r bytes
        const int a = r >> 2, b = r & 3;
        // rotate left by a dwords: t[d] = w[(d - a) & 3]
        uint32_t t0 = w.x, t1 = w.y, t2 = w.z, t3 = w.w;
        if (a & 2) { uint32_t u0 = t2, u1 = t3, u2 = t0, u3 = t1; t0 = u0; t1 = u1; t2 = u2; t3 = u3; }
        if (a & 1) { uint32_t u0 = t3, u1 = t0, u2 = t1, u3 = t2; t0 = u0; t1 = u1; t2 = u2; t3 = u3; }
        // rotate left by b bytes across the 128-bit ring
        const int sh = 32 - 8 * b;  // 32, 24, 16, 8
        w.x = (uint32_t)((((unsigned long long)t0 << 32) | t3) >> sh);
        w.y = (uint32_t)((((unsigned long long)t1 << 32) | t0) >> sh);
        w.z = (uint32_t)((((unsigned long long)t2 << 32) | t1) >> sh);
        w.w = (uint32_t)((((unsigned long long)t3 << 32) | t2) >> sh);
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

template <int Q, int Z, int SUB>
__global__ __launch_bounds__(256) void bcq_skinny_kernel(SkinnyParams p)
{
    __shared__ __attribute__((aligned(16))) uint8_t xs[2 * kXBufBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tg = blockIdx.x % p.ntg, part = blockIdx.x / p.ntg;
    const int tile = 4 * tg + wave;
    const bool active = tile < p.ntile;
    const int s_begin = (int)(((long long)part * p.nslice) / p.parts);
    const int s_end = (int)(((long long)(part + 1) * p.nslice) / p.parts);
    const int r = lane & 15, h = lane >> 4;
    const size_t slice_stride = (size_t)p.ntile * p.tile_bytes;
    const uint8_t *tile_ptr = p.blob + ((size_t)s_begin * p.ntile + (active ? tile : 0)) * p.tile_bytes;

    TileRegs<Q, Z, SUB> cur;
    if (active && s_begin < s_end) load_tile<Q, Z, SUB>(cur, tile_ptr, lane);
    {
        u32x4 xr[4];
        x_slice_load(p, s_begin, tid, xr);
        x_slice_store(xs, tid, xr);
    }
    __syncthreads();

    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};

    for (int slice = s_begin; slice < s_end; ++slice) {
        const bool more = slice + 1 < s_end;
        TileRegs<Q, Z, SUB> nxt;
        u32x4 xr[4];
        tile_ptr += slice_stride;
        if (more) {
            if (active) load_tile<Q, Z, SUB>(nxt, tile_ptr, lane);
            x_slice_load(p, slice + 1, tid, xr);
        }
        if (active) {
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
            const uint8_t *xb = xs + (slice - s_begin & 1) * kXBufBytes + r * kXPitchBytes + h * 256;
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
                    const f16x8 bx = *reinterpret_cast<const f16x8 *>(xb + (4 * dq + n) * 16);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
#pragma unroll
                        for (int i = 0; i < Q; ++i) {
                            f16x8 a;
                            if (n == 0) a = expand_byte<0>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                            if (n == 1) a = expand_byte<1>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                            if (n == 2) a = expand_byte<2>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                            if (n == 3) a = expand_byte<3>(w[t][i], w4[t][i], abs_pair[t][i][g]);
                            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bx, acc[t], 0, 0, 0);
                        }
                        if (Z) {
                            const u32x4 zz = {z_pair[t][g], z_pair[t][g], z_pair[t][g], z_pair[t][g]};
                            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, zz), bx, acc[t],
                                                                            0, 0, 0);
                        }
                    }
                }
            }
        }
        if (more) {
            x_slice_store(xs + (slice + 1 - s_begin & 1) * kXBufBytes, tid, xr);
            if (active) cur = nxt;
        }
        __syncthreads();  // next X slice written, everyone done reading the current one
    }

    if (!active) return;
    // acc[t][i] = partial of row 32*tile + 16*t + 4*h + i for batch column r
    const int col = r;
    if (col >= p.batch) return;
    if (p.parts == 1) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = tile * kTileRows + 16 * t + 4 * h + i;
                if (row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(acc[t][i]);
            }
        return;
    }
    unsigned long long mine[8], old[8];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tile * kTileRows + 16 * t + 4 * h + i;
            mine[4 * t + i] = encode_partial(acc[t][i]);
            old[4 * t + i] = __hip_atomic_fetch_add(p.accum + (size_t)col * p.Mp + row, mine[4 * t + i],
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tile * kTileRows + 16 * t + 4 * h + i;
            const unsigned long long total = old[4 * t + i] + mine[4 * t + i];
            if (arrivals_of(total) == (unsigned)p.parts) {
                if (row < p.M) p.Y[(size_t)col * p.ldy + row] = float_to_half_bits(decode_total(total));
                __hip_atomic_store(p.accum + (size_t)col * p.Mp + row, 0ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
int auto_skinny_parts(const Geom &g)
{
    // about 2000 waves in flight (8 per CU), at least one slice per part
    const int waves_per_part = ((g.ntile + 3) / 4) * 4;
    int parts = (2048 + waves_per_part / 2) / waves_per_part;
    if (parts < 1) parts = 1;
    if (parts > g.nslice) parts = g.nslice;
    return parts;
}

template <int Q, int Z, int SUB>
static hipError_t launch_skinny_one(const SkinnyParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL((bcq_skinny_kernel<Q, Z, SUB>), dim3((unsigned)(p.ntg * p.parts)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int Q, int Z>
static hipError_t launch_skinny_qz(const SkinnyParams &p, int sub, hipStream_t stream)
{
    if (sub == 2) return launch_skinny_one<Q, Z, 2>(p, stream);
    if (sub == 4) return launch_skinny_one<Q, Z, 4>(p, stream);
    return launch_skinny_one<Q, Z, 1>(p, stream);
}

hipError_t launch_skinny(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy,
                         int batch, void *workspace, int parts, hipStream_t stream)
{
    SkinnyParams p;
    p.blob = static_cast<const uint8_t *>(packed);
    p.X = X; p.Y = Y;
    p.accum = static_cast<unsigned long long *>(workspace);
    p.M = g.M; p.N = g.N; p.Mp = g.Mp; p.batch = batch; p.ldx = ldx; p.ldy = ldy;
    p.ntile = g.ntile; p.nslice = g.nslice; p.ntg = (g.ntile + 3) / 4;
    p.parts = parts > 0 ? parts : auto_skinny_parts(g);
    if (p.parts > g.nslice) p.parts = g.nslice;
    if (!workspace) p.parts = 1;  // only reachable for a single column slice
    p.tile_bytes = g.tile_bytes;
    switch (g.q * 2 + g.z) {
        case 2: return launch_skinny_qz<1, 0>(p, g.sub, stream);
        case 3: return launch_skinny_qz<1, 1>(p, g.sub, stream);
        case 4: return launch_skinny_qz<2, 0>(p, g.sub, stream);
        case 5: return launch_skinny_qz<2, 1>(p, g.sub, stream);
        case 6: return launch_skinny_qz<3, 0>(p, g.sub, stream);
        case 7: return launch_skinny_qz<3, 1>(p, g.sub, stream);
        case 8: return launch_skinny_qz<4, 0>(p, g.sub, stream);
        case 9: return launch_skinny_qz<4, 1>(p, g.sub, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace bcq
