// extern "C" entry points of libbcq: argument validation (host only, before any
// launch) and dispatch to the kernels.  See include/bcq.h for the contract.
#include <string.h>

#include "bcq_internal.h"

using namespace bcq;

namespace {

GemvTuning g_tuning;  // zeros = automatic

bool desc_ok(const bcq_desc *d, bcq_status *why)
{
    *why = BCQ_ERR_INVALID_ARG;
    if (!d) return false;
    if (d->M <= 0 || d->N <= 0 || d->N % 32 != 0) return false;
    if (d->q < 1 || d->group <= 0 || d->group % 32 != 0 || d->N % d->group != 0) return false;
    if (d->has_offset != 0 && d->has_offset != 1) return false;
    *why = BCQ_ERR_UNSUPPORTED;
    if (d->q > kMaxQ) return false;
    const bool one_scale_per_block = d->group % 128 == 0 || d->group == d->N;
    if (!(one_scale_per_block || d->group == 32 || d->group == 64)) return false;  // e.g. 96, 160
    if (((long long)d->N + kTileCols - 1) / kTileCols > kMaxSlices) return false;  // split-K arrival count is 10 bits
    // blob offsets are size_t; tile counts must fit int
    if ((long long)d->M + kTileRows > 0x7fffffffLL || (long long)d->N + kTileCols > 0x7fffffffLL) return false;
    *why = BCQ_OK;
    return true;
}

inline Geom geom_of(const bcq_desc *d) { return make_geom(d->M, d->N, d->q, d->group, d->has_offset); }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

size_t workspace_bytes(const Geom &g, int batch)
{
    return ws_bytes(g, batch);
}

}  // namespace

extern "C" {

size_t bcq_packed_bytes(const bcq_desc *desc)
{
    bcq_status why;
    if (!desc_ok(desc, &why)) return 0;
    Geom g = geom_of(desc);
    return (size_t)g.nslice * g.ntile * g.tile_bytes;
}

size_t bcq_workspace_bytes(const bcq_desc *desc, int32_t batch)
{
    bcq_status why;
    if (!desc_ok(desc, &why) || batch < 1 || batch > BCQ_MAX_BATCH) return 0;
    return workspace_bytes(geom_of(desc), batch);
}

bcq_status bcq_workspace_init(void *workspace, size_t bytes, void *stream)
{
    if (bytes == 0) return BCQ_OK;
    if (!workspace || !aligned(workspace, 16) || bytes % 4 != 0) return BCQ_ERR_INVALID_ARG;
    return launch_fill_zero(workspace, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? BCQ_OK
                                                                                             : BCQ_ERR_HIP;
}

bcq_status bcq_pack_rows(bcq_desc *desc, int32_t row_begin, int32_t rows, const uint8_t *codes,
                         const uint16_t *alpha, const uint16_t *offset, void *packed, void *stream)
{
    bcq_status why;
    if (!desc_ok(desc, &why)) return why;
    if (row_begin < 0 || rows <= 0 || (long long)row_begin + rows > desc->M) return BCQ_ERR_INVALID_ARG;
    if (!codes || !alpha || !packed) return BCQ_ERR_INVALID_ARG;
    if ((desc->has_offset != 0) != (offset != nullptr)) return BCQ_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(alpha, 2) || (offset && !aligned(offset, 2))) return BCQ_ERR_INVALID_ARG;
    if (launch_pack(geom_of(desc), row_begin, rows, codes, alpha, offset, packed,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
        return BCQ_ERR_HIP;
    desc->layout_version = BCQ_LAYOUT_VERSION;
    return BCQ_OK;
}

bcq_status bcq_pack(bcq_desc *desc, const uint8_t *codes, const uint16_t *alpha, const uint16_t *offset,
                    void *packed, void *stream)
{
    if (!desc) return BCQ_ERR_INVALID_ARG;
    return bcq_pack_rows(desc, 0, desc->M, codes, alpha, offset, packed, stream);
}

bcq_status bcq_from_linear(int32_t M, int32_t N, int32_t group, int32_t n_bits, int32_t q,
                           const int32_t *class_of_plane, const uint8_t *w_int, const float *S,
                           const float *qbias, uint8_t *codes, uint16_t *alpha, uint16_t *offset, void *stream)
{
    if (M <= 0 || N <= 0 || group <= 0 || N % group != 0) return BCQ_ERR_INVALID_ARG;
    if (n_bits < 1 || n_bits > 8 || q < 1 || q > n_bits || !class_of_plane) return BCQ_ERR_INVALID_ARG;
    if (q > kMaxQ) return BCQ_ERR_UNSUPPORTED;
    if (!w_int || !S || !qbias || !codes || !alpha || !offset) return BCQ_ERR_INVALID_ARG;
    if (!aligned(S, 4) || !aligned(qbias, 4) || !aligned(alpha, 2) || !aligned(offset, 2)) return BCQ_ERR_INVALID_ARG;
    bool seen[kMaxQ] = {false, false, false, false};
    for (int i = 0; i < n_bits; ++i) {
        if (class_of_plane[i] < 0 || class_of_plane[i] >= q) return BCQ_ERR_INVALID_ARG;
        seen[class_of_plane[i]] = true;
    }
    for (int c = 0; c < q; ++c)
        if (!seen[c]) return BCQ_ERR_INVALID_ARG;  // an empty class
    return launch_from_linear(M, N, group, n_bits, q, class_of_plane, w_int, S, qbias, codes, alpha, offset,
                              static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK
               : BCQ_ERR_HIP;
}

static bool quant_shape_ok(int32_t M, int32_t N, int32_t n_bits, int32_t q, bcq_status *why)
{
    *why = BCQ_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || N % 4 != 0 || n_bits < 2 || n_bits > 8 || q < 1 || q > n_bits) return false;
    *why = BCQ_ERR_UNSUPPORTED;
    if (q > kMaxQ || N > 32768) return false;
    *why = BCQ_OK;
    return true;
}

size_t bcq_quant_workspace_bytes(int32_t M, int32_t N)
{
    if (M <= 0 || N <= 0) return 0;
    return quant_workspace_bytes(M, N);
}

bcq_status bcq_quant_hessian(int32_t N, int32_t T, const float *X, float *H, void *stream)
{
    if (N <= 0 || T <= 0 || N % 4 != 0) return BCQ_ERR_INVALID_ARG;
    if (N > 32768) return BCQ_ERR_UNSUPPORTED;
    if (!X || !H || !aligned(X, 16) || !aligned(H, 16)) return BCQ_ERR_INVALID_ARG;
    return launch_quant_hessian(N, T, X, H, static_cast<hipStream_t>(stream)) == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
}

size_t bcq_quant_factor_workspace_bytes(int32_t N)
{
    if (N <= 0 || N % 4 != 0 || N > 32768) return 0;
    return quant_factor_workspace_bytes(N);
}

bcq_status bcq_quant_factor(int32_t N, float damp, const float *H, float *U, void *workspace, void *stream)
{
    if (N <= 0 || N % 4 != 0 || !(damp >= 0.0f)) return BCQ_ERR_INVALID_ARG;
    if (N > 32768) return BCQ_ERR_UNSUPPORTED;
    if (!H || !U || !aligned(H, 16) || !aligned(U, 16)) return BCQ_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 16)) return BCQ_ERR_WORKSPACE;
    return launch_quant_factor(N, damp, H, U, workspace, static_cast<hipStream_t>(stream)) == hipSuccess ? BCQ_OK
                                                                                                       : BCQ_ERR_HIP;
}

bcq_status bcq_quant_search(int32_t M, int32_t N, int32_t n_bits, int32_t q, int32_t grid, const float *W,
                            const float *H, float *S, float *qbias, int8_t *class_of_plane, float *err,
                            void *workspace, void *stream)
{
    bcq_status why;
    if (!quant_shape_ok(M, N, n_bits, q, &why)) return why;
    if (grid < 1 || grid > 4096) return BCQ_ERR_INVALID_ARG;
    if (!W || !H || !S || !qbias || !class_of_plane) return BCQ_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 16)) return BCQ_ERR_WORKSPACE;
    if (!aligned(W, 4) || !aligned(H, 16) || !aligned(S, 4) || !aligned(qbias, 4) || (err && !aligned(err, 4)))
        return BCQ_ERR_INVALID_ARG;
    return launch_quant_search(M, N, n_bits, q, grid, W, H, S, qbias, class_of_plane, err, workspace,
                               static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK
               : BCQ_ERR_HIP;
}

bcq_status bcq_quant_gptq(int32_t M, int32_t N, int32_t n_bits, int32_t q, const float *W, const float *U,
                          const float *S, const float *qbias, const int8_t *class_of_plane, uint8_t *w_int,
                          void *workspace, void *stream)
{
    bcq_status why;
    if (!quant_shape_ok(M, N, n_bits, q, &why)) return why;
    if (!W || !U || !S || !qbias || !class_of_plane || !w_int) return BCQ_ERR_INVALID_ARG;
    if (!workspace || !aligned(workspace, 16)) return BCQ_ERR_WORKSPACE;
    if (!aligned(W, 4) || !aligned(U, 16) || !aligned(S, 4) || !aligned(qbias, 4)) return BCQ_ERR_INVALID_ARG;
    return launch_quant_gptq(M, N, n_bits, q, W, U, S, qbias, class_of_plane, w_int, workspace,
                             static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK
               : BCQ_ERR_HIP;
}

bcq_status bcq_from_linear_rows(int32_t M, int32_t N, int32_t n_bits, int32_t q, const int8_t *class_of_plane,
                                const uint8_t *w_int, const float *S, const float *qbias, uint8_t *codes,
                                uint16_t *alpha, uint16_t *offset, void *stream)
{
    bcq_status why;
    if (!quant_shape_ok(M, N, n_bits, q, &why)) return why;
    if (!class_of_plane || !w_int || !S || !qbias || !codes || !alpha || !offset) return BCQ_ERR_INVALID_ARG;
    if (!aligned(S, 4) || !aligned(qbias, 4) || !aligned(alpha, 2) || !aligned(offset, 2)) return BCQ_ERR_INVALID_ARG;
    return launch_from_linear_rows(M, N, n_bits, q, class_of_plane, w_int, S, qbias, codes, alpha, offset,
                                   static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK
               : BCQ_ERR_HIP;
}

bcq_status bcq_unpack(const bcq_desc *desc, const void *packed, uint8_t *codes, uint16_t *alpha,
                      uint16_t *offset, void *stream)
{
    bcq_status why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->layout_version != BCQ_LAYOUT_VERSION) return BCQ_ERR_INVALID_ARG;
    if (!packed || !aligned(packed, 256)) return BCQ_ERR_INVALID_ARG;
    if (offset && !desc->has_offset) return BCQ_ERR_INVALID_ARG;
    if ((alpha && !aligned(alpha, 2)) || (offset && !aligned(offset, 2))) return BCQ_ERR_INVALID_ARG;
    if (launch_unpack(geom_of(desc), packed, codes, alpha, offset, static_cast<hipStream_t>(stream)) != hipSuccess)
        return BCQ_ERR_HIP;
    return BCQ_OK;
}

bcq_status bcq_gemm_skinny(const bcq_desc *desc, const void *packed, const uint16_t *X, int32_t ldx,
                           uint16_t *Y, int32_t ldy, int32_t batch, void *workspace, void *stream)
{
    bcq_status why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->layout_version != BCQ_LAYOUT_VERSION) return BCQ_ERR_INVALID_ARG;
    if (batch < 1 || batch > BCQ_MAX_BATCH) return BCQ_ERR_INVALID_ARG;
    if (!packed || !X || !Y) return BCQ_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(X, 16) || !aligned(Y, 2)) return BCQ_ERR_INVALID_ARG;
    if (ldx < desc->N || ldy < desc->M || ldx % 8 != 0) return BCQ_ERR_INVALID_ARG;
    Geom g = geom_of(desc);
    if (workspace_bytes(g, batch) > 0 && (!workspace || !aligned(workspace, 16))) return BCQ_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // batch 1: the table-lookup GEMV (HBM-bound); batch >= 2: the matrix-core kernel, weights read once
    hipError_t e = batch == 1 ? launch_gemv(g, packed, X, Y, workspace, g_tuning, s)
                              : launch_skinny(g, packed, X, ldx, Y, ldy, batch, workspace, g_tuning, s);
    return e == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
}

bcq_status bcq_gemv(const bcq_desc *desc, const void *packed, const uint16_t *x, uint16_t *y, void *workspace,
                    void *stream)
{
    if (!desc) return BCQ_ERR_INVALID_ARG;
    return bcq_gemm_skinny(desc, packed, x, desc->N, y, desc->M, 1, workspace, stream);
}

bcq_status bcq_gemv_noalloc(const bcq_desc *desc, const void *packed, const uint16_t *x, uint16_t *y, void *stream)
{
    bcq_status why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->layout_version != BCQ_LAYOUT_VERSION) return BCQ_ERR_INVALID_ARG;
    if (!packed || !x || !y) return BCQ_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(x, 16) || !aligned(y, 2)) return BCQ_ERR_INVALID_ARG;
    const Geom g = geom_of(desc);
    if (g.Mp > kStaticScratchRows) return BCQ_ERR_SCRATCH_LIMIT;  // more rows than the static array holds
    hipStream_t s = static_cast<hipStream_t>(stream);
    void *ws = nullptr;
    const size_t need = workspace_bytes(g, 1);
    if (need > 0) {
        if (static_scratch(&ws) != hipSuccess) return BCQ_ERR_HIP;
        // the array keeps whatever the last call on this GPU left (zeros, unless that call was cut short):
        // clear the part this call uses, with a kernel rather than a memset node (the caller may be capturing)
        if (launch_fill_zero(ws, need, s) != hipSuccess) return BCQ_ERR_HIP;
    }
    return launch_gemv(g, packed, x, y, ws, g_tuning, s) == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
}

size_t bcq_read_probe_sink_bytes(void) { return (size_t)kProbeBlocks * 4; }

bcq_status bcq_read_probe(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink || bytes == 0 || bytes % 16 != 0 || !aligned(buf, 16) || !aligned(sink, 4))
        return BCQ_ERR_INVALID_ARG;
    return launch_read_probe(buf, bytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? BCQ_OK
                                                                                              : BCQ_ERR_HIP;
}

bcq_status bcq_set_option(const char *name, int32_t value)
{
    if (!name || value < 0) return BCQ_ERR_INVALID_ARG;
    if (strcmp(name, "workgroups") == 0) {
        g_tuning.workgroups = value;
        return BCQ_OK;
    }
    if (strcmp(name, "waves") == 0 && (value == 0 || value == 4 || value == 8)) {
        g_tuning.waves = value;
        return BCQ_OK;
    }
    if (strcmp(name, "gemv_early") == 0 && value <= 2) {
        g_tuning.early = value;
        return BCQ_OK;
    }
    if (strcmp(name, "skinny_parts") == 0) {
        g_tuning.skinny_parts = value;
        return BCQ_OK;
    }
    if (strcmp(name, "skinny_version") == 0 && value <= 6) {
        g_tuning.skinny_version = value;
        return BCQ_OK;
    }
    if (strcmp(name, "skinny_lds_steps") == 0 && (value == 0 || value == 3 || value == 4)) {
        g_tuning.skinny_lds_steps = value;
        return BCQ_OK;
    }
    return BCQ_ERR_INVALID_ARG;
}

const char *bcq_status_string(bcq_status status)
{
    switch (status) {
        case BCQ_OK: return "ok";
        case BCQ_ERR_INVALID_ARG: return "invalid argument";
        case BCQ_ERR_UNSUPPORTED: return "unsupported configuration";
        case BCQ_ERR_WORKSPACE: return "workspace missing or misaligned";
        case BCQ_ERR_HIP: return "HIP runtime error";
        case BCQ_ERR_SCRATCH_LIMIT: return "more rows than the library's static scratch buffer holds";
    }
    return "unknown status";
}

}  // extern "C"
