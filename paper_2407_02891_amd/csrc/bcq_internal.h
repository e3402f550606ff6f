// Internal declarations shared by the translation units of libbcq (not public).
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/bcq.h"
#include "bcq_layout.h"

namespace bcq {

// Launchers; each returns the hipError_t of its last launch.
// Packs the rows [row0, row0 + rows) of the layer; the sources hold only those rows.
hipError_t launch_pack(const Geom &g, int row0, int rows, const uint8_t *codes, const uint16_t *alpha,
                       const uint16_t *offset, void *packed, hipStream_t stream);
hipError_t launch_unpack(const Geom &g, const void *packed, uint8_t *codes, uint16_t *alpha,
                         uint16_t *offset, hipStream_t stream);
hipError_t launch_fill_zero(void *ptr, size_t bytes, hipStream_t stream);
// Linear n-bit integers + per-group scale/bias + plane tying -> codes, fused alpha, fused offset
// (Eq. 6, 9-11).  hipErrorInvalidValue if the tying is malformed.
hipError_t launch_from_linear(int M, int N, int group, int n_bits, int q, const int32_t *class_of_plane,
                              const uint8_t *w_int, const float *S, const float *qbias, uint8_t *codes,
                              uint16_t *alpha, uint16_t *offset, hipStream_t stream);
// The quantiser (row-wise parameters): search over scales and plane tyings, GPTQ pass, fusion.
size_t quant_workspace_bytes(int M, int N);
size_t quant_factor_workspace_bytes(int N);
hipError_t launch_quant_factor(int N, float damp, const float *H, float *U, void *workspace, hipStream_t stream);
hipError_t launch_quant_hessian(int N, int T, const float *X, float *H, hipStream_t stream);
hipError_t launch_quant_search(int M, int N, int n_bits, int q, int grid, const float *W, const float *H, float *S,
                               float *qbias, int8_t *labels, float *err_out, void *workspace, hipStream_t stream);
hipError_t launch_quant_gptq(int M, int N, int n_bits, int q, const float *W, const float *U, const float *S,
                             const float *qbias, const int8_t *labels, uint8_t *w_int, void *workspace,
                             hipStream_t stream);
hipError_t launch_from_linear_rows(int M, int N, int n_bits, int q, const int8_t *labels, const uint8_t *w_int,
                                   const float *S, const float *qbias, uint8_t *codes, uint16_t *alpha,
                                   uint16_t *offset, hipStream_t stream);
struct ConvertPlan;
bool make_convert_plan(int n_bits, int q, const int32_t *class_of_plane, ConvertPlan *plan);
// Launch shape of the GEMV (bcq_set_option); zeros mean "choose automatically".
struct GemvTuning {
    int workgroups = 0; // grid size
    int waves = 0;      // waves per workgroup: 4 or 8
    int early = 0;      // GEMV: 1 = build the tables before the first tile has arrived, 2 = never, 0 = automatic
    void *trace = nullptr;  // tracing build only: DEVICE buffer of kTraceSlots words per wave of the grid
    int trace_groups = 0;   // tracing build, skinny kernel: workgroups that buffer has room for (8 waves each)
    int skinny_parts = 0;  // K split of the skinny kernel
    int skinny_version = 0;    // 1 = the first skinny kernel (alpha folded into A) also where the second applies,
                               // 3 = the table kernel for up to four vectors where it applies, 4 = never that one,
                               // 5 = the two-vector table kernel where it applies, 6 = never that one
    int skinny_lds_steps = 0;  // second skinny kernel: MFMA steps per block whose A operand comes from the
                               // LDS table, 3 or 4 (0 = automatic = 4)
};
hipError_t launch_gemv(const Geom &g, const void *packed, const uint16_t *x, uint16_t *y,
                       void *workspace, const GemvTuning &tuning, hipStream_t stream);
// Single-pass kernel for 2 <= batch <= 16 (matrix cores); parts = K split, 0 = automatic.
hipError_t launch_skinny(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy,
                         int batch, void *workspace, const GemvTuning &tuning, hipStream_t stream);
// Sign-sum tables holding four activation vectors side by side (bcq_lut4.hip): 2 <= batch <= 4.
bool lut4_applies(const Geom &g, int batch, const void *workspace);
hipError_t launch_lut4(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy, int batch,
                       void *workspace, const GemvTuning &tuning, hipStream_t stream);
// The GEMV's tables with both vectors of a two-vector call side by side (bcq_gemv2.hip): batch == 2.
bool gemv2_applies(const Geom &g, int batch, const void *workspace);
hipError_t launch_gemv2(const Geom &g, const void *packed, const uint16_t *X, int ldx, uint16_t *Y, int ldy,
                        void *workspace, const GemvTuning &tuning, hipStream_t stream);
hipError_t launch_read_probe(const void *buf, size_t bytes, void *sink, hipStream_t stream);

// Rows the file-scope split-K scratch array covers (bcq_gemv_noalloc): 1 MiB per GPU.
constexpr int kStaticScratchRows = 131072;
// Device address of the current device's copy of that array (asked from the runtime on first use).
hipError_t static_scratch(void **ptr);

constexpr int kProbeBlocks = 512;  // the GEMV's grid: two workgroups per CU

constexpr int kTraceSlots = 16;  // words per wave in the tracing build's timeline buffer

// Launch shape of the GEMV for a layer under given overrides (what launch_gemv will use).
void gemv_launch_shape(const Geom &g, const GemvTuning &tuning, int *workgroups, int *waves, bool *early);

// Grid size the GEMV uses when none is forced.
int auto_workgroups(const Geom &g, int waves_per_group);

}  // namespace bcq
