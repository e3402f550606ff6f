/*
 * bcq.h -- C ABI of the MI355X (gfx950) binary-coding matrix-vector library.
 *
 * The operation is the inference form of GPTQT (arXiv 2407.02891): a linear
 * layer whose weight is stored as q bit-planes of signs with per-group scales
 * and an optional per-group offset (paper Eq. 3, dequantisation line, and
 * Eq. 11, the fused form):
 *
 *     W[m][k] = sum_{i<q} alpha[m][k/group][i] * s_i[m][k]  (+ offset[m][k/group])
 *     y[m]    = sum_k W[m][k] * x[k]                        s_i in {-1,+1}
 *
 * evaluated directly on the planes, never materialising W (Sec. II-D, last
 * paragraph; Sec. III "Speed up of GPTQT").  Activations and outputs are IEEE
 * binary16 (the paper keeps activations at fp16); accumulation is fp32; the
 * result is rounded to binary16 to nearest-even.
 *
 * Conventions for every entry point
 *   - plain C types only; a hipStream_t is passed as void* (NULL = the null
 *     stream); every pointer marked DEVICE must be device memory of the
 *     current HIP device, every pointer marked HOST is ordinary host memory;
 *   - the caller owns every buffer; the library never allocates, frees or
 *     synchronises; work is enqueued on the given stream and the call returns;
 *   - all argument checks happen on the host before any launch; a failed
 *     check launches nothing and returns a status other than BCQ_OK;
 *   - binary16 values travel as uint16_t bit patterns.
 */
#ifndef BCQ_H
#define BCQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BCQ_OK = 0,
    BCQ_ERR_INVALID_ARG = 1, /* NULL pointer, bad size, misalignment, bad batch     */
    BCQ_ERR_UNSUPPORTED = 2, /* well-formed request outside what the kernels cover  */
    BCQ_ERR_WORKSPACE = 3,   /* workspace missing where bcq_workspace_bytes() > 0   */
    BCQ_ERR_HIP = 4,         /* the HIP runtime reported an error at launch         */
    BCQ_ERR_SCRATCH_LIMIT = 5 /* bcq_gemv_noalloc: more rows than BCQ_NOALLOC_MAX_ROWS */
} bcq_status;

/* Version of the opaque packed layout written by bcq_pack. */
#define BCQ_LAYOUT_VERSION 2

/* Most output rows (after padding to a multiple of 32) bcq_gemv_noalloc accepts. */
#define BCQ_NOALLOC_MAX_ROWS 131072

/* Largest batch bcq_gemm_skinny accepts. */
#define BCQ_MAX_BATCH 64

/*
 * Problem descriptor (HOST, plain data, filled by the caller).
 *   M, N        out rows, in columns; N must be a multiple of 32 and at most
 *               523776 (larger N is BCQ_ERR_UNSUPPORTED)
 *   q           number of sign planes, 1..4 (the paper uses 2 and 3)
 *   group       columns sharing one alpha per plane (and one offset); must
 *               divide N and be 32, 64, a multiple of 128, or N itself (any N).
 *               group == N gives the paper's row-wise parameters (Sec. II-A:
 *               quantisation parameters are fixed per row).  Other multiples
 *               of 32 (96, 160, ...) are well-formed but BCQ_ERR_UNSUPPORTED.
 *   has_offset  1 if the fused offset term of Eq. 11, (2^n-1)/2*S + qbias, is
 *               present, else 0
 *   layout_version  set by bcq_pack; bcq_gemv / bcq_gemm_skinny / bcq_unpack
 *               refuse a descriptor whose value is not BCQ_LAYOUT_VERSION
 */
typedef struct bcq_desc {
    int32_t M, N;
    int32_t q;
    int32_t group;
    int32_t has_offset;
    int32_t layout_version;
} bcq_desc;

/* Size in bytes of the opaque packed weight blob for this descriptor
 * (0 if the descriptor is invalid).  HOST-only computation. */
size_t bcq_packed_bytes(const bcq_desc *desc);

/* Size in bytes of the workspace bcq_gemv (batch = 1) or bcq_gemm_skinny needs
 * (0 if the descriptor or batch is invalid, or if N <= 512, where no split
 * over columns happens).  It holds one 64-bit split-K accumulator per row and
 * batch column.  HOST-only computation. */
size_t bcq_workspace_bytes(const bcq_desc *desc, int32_t batch);

/*
 * Zero a workspace.  Required once before its first use; bcq_gemv and
 * bcq_gemm_skinny leave every accumulator zero again when they finish, so one
 * workspace can serve any sequence of calls on ONE stream (calls sharing a
 * workspace must not overlap in time).  Uses a fill kernel, not a memset node,
 * so it may be captured into a graph.
 *   workspace DEVICE, 16-byte aligned; bytes a multiple of 4.
 */
bcq_status bcq_workspace_init(void *workspace, size_t bytes, void *stream);

/*
 * Integer weights + scales -> packed bit-planes (Eq. 11 operands).
 *   codes  DEVICE [M][N] uint8: bit i of codes[m*N+k] is the sign of plane i
 *          for weight (m,k): 1 means +1, 0 means -1 (the paper leaves the
 *          encoding open); bits >= q are ignored
 *   alpha  DEVICE [M][N/group][q] binary16
 *   offset DEVICE [M][N/group] binary16, or NULL iff desc->has_offset == 0
 *   packed DEVICE, bcq_packed_bytes(desc) bytes, 256-byte aligned; opaque
 * Sets desc->layout_version.  Offline step, not part of the timed path.
 */
bcq_status bcq_pack(bcq_desc *desc, const uint8_t *codes, const uint16_t *alpha,
                    const uint16_t *offset, void *packed, void *stream);

/*
 * Result of the paper's two-step quantiser -> operands of bcq_pack (Sec. II-B Eq. 6, Sec. II-D
 * Eq. 8-11).  The quantiser leaves n_bits-bit linear integers W_int, one scale S and one bias
 * qbias per scaling group (W_hat = S * W_int + qbias), and a tying of the n_bits linear
 * bit-planes into q classes that share one sign each (Eq. 10 ties planes 2 and 3 of three).
 *   class_of_plane HOST [n_bits]: class (0..q-1) of linear plane i+1, i.e. of bit i of W_int,
 *                  whose weight in Eq. 9 is 2^(i-1); every class must be non-empty
 *   w_int   DEVICE [M][N] uint8, values 0 .. 2^n_bits - 1 (higher bits ignored)
 *   S, qbias DEVICE [M][N/group] binary32
 *   codes   DEVICE [M][N] uint8 out: bit o = sign of fused plane o (1 means +1)
 *   alpha   DEVICE [M][N/group][q] binary16 out: S * alpha_hat_o, alpha_hat_o = sum of 2^(i-1)
 *           over the bits i tied into plane o; planes ordered by descending alpha_hat
 *   offset  DEVICE [M][N/group] binary16 out: (2^n_bits - 1)/2 * S + qbias
 * Every W_int is first replaced by the nearest integer the tying can represent (Eq. 6; a tie
 * goes to the smaller one), so integers already in that set pass unchanged.  alpha and offset
 * are evaluated in binary64 and rounded once to binary16 (nearest even).  Use has_offset = 1
 * in the descriptor given to bcq_pack.  Offline step.
 */
bcq_status bcq_from_linear(int32_t M, int32_t N, int32_t group, int32_t n_bits, int32_t q,
                           const int32_t *class_of_plane, const uint8_t *w_int, const float *S,
                           const float *qbias, uint8_t *codes, uint16_t *alpha, uint16_t *offset,
                           void *stream);

/*
 * The quantiser itself, for one layer with row-wise parameters (Sec. II-A Eq. 1-2, Sec. II-B Eq. 5-6,
 * Sec. II-C Eq. 7 and the algorithm closing Sec. II-D).  Offline tooling, in steps:
 *
 *   bcq_quant_hessian  H += 2 X^T X for T more calibration inputs X [T][N] (Sec. II-A: H = 2 X X^T with the
 *                      paper's X = inputs as columns); H DEVICE [N][N] in/out, zero it before the first batch;
 *                      X and H binary32, 16-byte aligned.  Optional: H may come from anywhere.
 *   bcq_quant_factor   U = the upper triangular factor with (H + damp * mean(diag H) * I)^-1 = U^T U, in binary32
 *                      (H is not modified; needs H positive definite after dampening, otherwise U holds NaNs);
 *                      workspace DEVICE, bcq_quant_factor_workspace_bytes(N) bytes, 16-byte aligned, no init.
 *                      Optional: U may come from any linear-algebra library.
 *   bcq_quant_search   per row: qbias = min w; the scale S' on `grid` equidistant points inside
 *                      ((max-min)/(2^(n_bits+1)-1), (max-min)/(2^(n_bits-1)-1)) (Eq. 7) and the tying
 *                      of the n_bits linear planes into q classes (Eq. 10) that minimise the output
 *                      error d (H/2) d^T of the row, d = S' W_q + qbias - w, W_q = nearest
 *                      representable integer of clamp(rne((w - qbias)/S')) (Eq. 5, 6).  Candidates
 *                      are visited scale-major, tyings in lexicographic order of their classes; the
 *                      first with the smallest error wins.
 *   bcq_quant_gptq     the column-by-column pass with error compensation (Eq. 1-2) using those
 *                      parameters; U is the upper Cholesky factor of the inverse (dampened) Hessian,
 *                      H^-1 = U^T U (bcq_quant_factor, or any linear-algebra library).
 *   bcq_from_linear_rows   bcq_from_linear with one tying per row and one scaling group per row
 *                      (use group = N and has_offset = 1 for bcq_pack).
 *
 *   W   DEVICE [M][N] binary32 weights (not modified)
 *   H   DEVICE [N][N] binary32, 2 X X^T of the calibration inputs, symmetric (bcq_quant_search reads only its
 *       upper triangle), 16-byte aligned
 *   U   DEVICE [N][N] binary32, upper triangular, 16-byte aligned
 *   S, qbias DEVICE [M] binary32 (out of search, in of the others)
 *   class_of_plane DEVICE [M][n_bits] int8: class (0..q-1) of bit i of row m (out of search)
 *   err DEVICE [M] binary32 or NULL: the smallest error found (out)
 *   w_int DEVICE [M][N] uint8: integers in the row's representable set (out of gptq)
 *   codes DEVICE [M][N] uint8, alpha DEVICE [M][q] binary16, offset DEVICE [M] binary16 (out)
 *   workspace DEVICE, bcq_quant_workspace_bytes(M, N) bytes, 16-byte aligned (scratch, no init)
 * N a multiple of 4, 2 <= n_bits <= 8, q <= n_bits, 1 <= grid <= 4096; q > 4 or N > 32768 is
 * BCQ_ERR_UNSUPPORTED (all three calls).
 * Integer decisions are taken in binary64; the error sums and the compensation run in binary32
 * on the matrix cores (v_mfma_f32_32x32x2_f32).
 */
size_t bcq_quant_workspace_bytes(int32_t M, int32_t N);
bcq_status bcq_quant_hessian(int32_t N, int32_t T, const float *X, float *H, void *stream);
size_t bcq_quant_factor_workspace_bytes(int32_t N);
bcq_status bcq_quant_factor(int32_t N, float damp, const float *H, float *U, void *workspace, void *stream);
bcq_status bcq_quant_search(int32_t M, int32_t N, int32_t n_bits, int32_t q, int32_t grid, const float *W,
                            const float *H, float *S, float *qbias, int8_t *class_of_plane, float *err,
                            void *workspace, void *stream);
bcq_status bcq_quant_gptq(int32_t M, int32_t N, int32_t n_bits, int32_t q, const float *W, const float *U,
                          const float *S, const float *qbias, const int8_t *class_of_plane, uint8_t *w_int,
                          void *workspace, void *stream);
bcq_status bcq_from_linear_rows(int32_t M, int32_t N, int32_t n_bits, int32_t q, const int8_t *class_of_plane,
                                const uint8_t *w_int, const float *S, const float *qbias, uint8_t *codes,
                                uint16_t *alpha, uint16_t *offset, void *stream);

/*
 * bcq_pack for a range of rows: writes the rows [row_begin, row_begin + rows) of the layer
 * `desc` describes from sources that hold ONLY those rows (codes [rows][N], alpha
 * [rows][N/group][q], offset [rows][N/group]).  Layers that are applied to the same
 * activations (the q/k/v projections of an attention block, the gate/up projections of a
 * gated MLP) can so be packed from their own tensors into one blob with M = the sum of their
 * rows, and then cost ONE bcq_gemv / bcq_gemm_skinny: one launch, one staging of the
 * activations, y = the concatenation of their outputs (Eq. 11 is row-wise, so stacking rows
 * changes no result).  Every row of the layer must be covered by some call before the blob is
 * used; the call that covers the last row also writes the padding.  Calls for disjoint row
 * ranges may run concurrently.  Sets desc->layout_version.
 */
bcq_status bcq_pack_rows(bcq_desc *desc, int32_t row_begin, int32_t rows, const uint8_t *codes,
                         const uint16_t *alpha, const uint16_t *offset, void *packed, void *stream);

/* Inverse of bcq_pack (for tests): any of codes / alpha / offset may be NULL
 * to skip that output.  All DEVICE. */
bcq_status bcq_unpack(const bcq_desc *desc, const void *packed, uint8_t *codes,
                      uint16_t *alpha, uint16_t *offset, void *stream);

/*
 * y[M] = W_q x[N]  (batch 1; paper Eq. 11 applied to one activation vector).
 *   packed    DEVICE, written by bcq_pack for the same descriptor
 *   x         DEVICE [N] binary16, 16-byte aligned
 *   y         DEVICE [M] binary16, 2-byte aligned
 *   workspace DEVICE, bcq_workspace_bytes(desc, 1) bytes, 16-byte aligned,
 *             initialised once with bcq_workspace_init; may be NULL only if
 *             that size is 0
 * Resolution of the split over columns (N > 512): every 512-column slice hands its fp32 partial sum of
 * a row over as a multiple of 2^-34 (5.8e-11), so a result carries an absolute error of at most
 * ceil(N/512) * 2^-35 on top of the fp32 rounding, whatever its size.  Against the 2e-3 relative
 * tolerance (measured on max(|y|, rms(y)/64)) that is negligible as long as rms(y) >= 1e-6 *
 * ceil(N/512); layers whose outputs are all smaller than that should be rescaled by the caller (alpha is
 * linear in y).  Inputs must be finite: a non-finite activation gives unspecified output values.
 */
bcq_status bcq_gemv(const bcq_desc *desc, const void *packed, const uint16_t *x,
                    uint16_t *y, void *workspace, void *stream);

/*
 * bcq_gemv without a workspace argument, for callers that cannot allocate device memory or size
 * buffers at run time (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc).  Same kernels and same result, bit for bit, as bcq_gemv; the split-K accumulators
 * live in a static device array inside the library (8 bytes x BCQ_NOALLOC_MAX_ROWS = 1 MiB on
 * every GPU the library is used on, held until the process ends).  The call allocates nothing and
 * frees nothing: it looks up the array's device address (asked from the HIP runtime on the first
 * call on each device, with that device current), clears the part it needs with a fill kernel and
 * launches the GEMV, all on `stream`.  Rows beyond BCQ_NOALLOC_MAX_ROWS (M rounded up to 32) are
 * refused with BCQ_ERR_SCRATCH_LIMIT before anything is launched.  All calls on one GPU share the
 * one array: calls that overlap in time on the same GPU (different streams, or graph branches)
 * race; serialise them.  packed, x, y as for bcq_gemv.
 */
bcq_status bcq_gemv_noalloc(const bcq_desc *desc, const void *packed, const uint16_t *x,
                            uint16_t *y, void *stream);

/*
 * Y[j][m] = sum_k W_q[m][k] X[j][k],  1 <= batch <= BCQ_MAX_BATCH (64): the fused form of Eq. 11 applied
 * to `batch` activation vectors at once (the paper measures batch 1 only, Sec. III "Speed up of GPTQT", and
 * names larger batches as the method's limitation, Sec. IV).  The weights are read once
 * per call with groups that are multiples of 128 (or N), and once per 16 batch columns with
 * groups of 32/64.
 *   X   DEVICE, row j starts at X + j*ldx (elements), ldx >= N, ldx % 8 == 0
 *   Y   DEVICE, row j starts at Y + j*ldy (elements), ldy >= M
 *   workspace as for bcq_gemv with bcq_workspace_bytes(desc, batch)
 */
bcq_status bcq_gemm_skinny(const bcq_desc *desc, const void *packed,
                           const uint16_t *X, int32_t ldx, uint16_t *Y,
                           int32_t ldy, int32_t batch, void *workspace,
                           void *stream);

/*
 * Streaming-read probe: reads `bytes` (a multiple of 16) of DEVICE memory with
 * the same 128-bit coalesced loads and launch shape the GEMV uses and writes a
 * 4-byte checksum per workgroup to `sink` (DEVICE, at least
 * bcq_read_probe_sink_bytes() bytes).  It measures the read bandwidth the
 * chip can reach, the ceiling against which the GEMV's rate is reported.
 */
size_t bcq_read_probe_sink_bytes(void);
bcq_status bcq_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

/*
 * Launch-shape overrides for tuning runs (HOST state, process-wide, not
 * thread-safe).  Names: "workgroups" (grid size of the GEMV and of the skinny
 * kernel), "waves" (waves per workgroup, 4 or 8: the GEMV, the table kernel of
 * bcq_gemm_skinny up to 16 columns and its 32-column pass), "gemv_early" (1 = the GEMV
 * builds its tables before its first tile has arrived, 2 = never; automatic: when no wave has
 * more than one tile), "skinny_parts" (K
 * split of bcq_gemm_skinny for batch >= 2), "skinny_version" (1 = the kernel
 * that folds alpha into the matrix-core operand, 2 = the kernel that takes +-1
 * operands from an LDS table, with q = 4 at most 32 columns per pass; groups of
 * 32/64 always use 1; 3 = for batch 2..4 the kernel with sign-sum tables of four
 * vectors wherever it applies, 4 = never that one; 5 = for batch 2 the GEMV's table kernel
 * with two vectors per table entry wherever it applies, 6 = never that one, the others chosen
 * automatically), "skinny_lds_steps" (3 or 4, kernel 2 only); 0 =
 * automatic.
 * Unknown names or values return BCQ_ERR_INVALID_ARG.
 */
bcq_status bcq_set_option(const char *name, int32_t value);

/* Static, NUL-terminated description of a status code. */
const char *bcq_status_string(bcq_status status);

#ifdef __cplusplus
}
#endif
#endif /* BCQ_H */
