// Entry points of the tracing build of the GEMV and the skinny GEMM (libbcq_trace.so; built by build.py
// --trace from bcq_gemv.hip and bcq_skinny.hip compiled with -DBCQ_TRACE, bcq_pack.hip and this file; used
// by trace_gemv.py).  A diagnostic, not part of the product library: same kernels, plus time stamps per wave.
#ifndef BCQ_TRACE
#error "this file belongs to the tracing build (-DBCQ_TRACE)"
#endif
#include "bcq_internal.h"

using namespace bcq;

extern "C" {

// Launch shape the traced call will use: workgroups, waves per workgroup, early table build (0/1).
int bcq_gemv_trace_shape(const bcq_desc *d, int32_t workgroups_opt, int32_t waves_opt, int32_t early_opt,
                         int32_t *workgroups, int32_t *waves, int32_t *early)
{
    if (!d || !workgroups || !waves || !early) return 1;
    GemvTuning t;
    t.workgroups = workgroups_opt;
    t.waves = waves_opt;
    t.early = early_opt;
    int groups, nw;
    bool e;
    gemv_launch_shape(make_geom(d->M, d->N, d->q, d->group, d->has_offset), t, &groups, &nw, &e);
    *workgroups = groups;
    *waves = nw;
    *early = e ? 1 : 0;
    return 0;
}

// bcq_gemv with a timeline: trace = DEVICE buffer of workgroups * waves * 16 uint32 (see trace_gemv.py for
// the meaning of the slots).  No argument checks beyond NULL: a diagnostic for the library's own tests.
int bcq_gemv_trace(const bcq_desc *d, const void *packed, const uint16_t *x, uint16_t *y, void *workspace,
                   void *trace, int32_t workgroups_opt, int32_t waves_opt, int32_t early_opt, void *stream)
{
    if (!d || !packed || !x || !y || !trace) return 1;
    const Geom g = make_geom(d->M, d->N, d->q, d->group, d->has_offset);
    GemvTuning t;
    t.workgroups = workgroups_opt;
    t.waves = waves_opt;
    t.early = early_opt;
    t.trace = trace;
    return launch_gemv(g, packed, x, y, workspace, t, static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : 4;
}

// bcq_gemm_skinny with a timeline (table kernel, batch <= 16, one scaling group per block): trace = DEVICE
// buffer of trace_groups * 8 * 16 uint32, zeroed by the caller; workgroup w, wave v writes record 8 w + v
// whatever the number of waves per workgroup (4 or 8).
int bcq_skinny_trace(const bcq_desc *d, const void *packed, const uint16_t *X, int32_t ldx, uint16_t *Y, int32_t ldy,
                     int32_t batch, void *workspace, void *trace, int32_t trace_groups, int32_t waves_opt, void *stream)
{
    if (!d || !packed || !X || !Y || !trace || !workspace || batch < 2 || batch > 16 || trace_groups < 1) return 1;
    const Geom g = make_geom(d->M, d->N, d->q, d->group, d->has_offset);
    if (g.sub != 1) return 1;
    GemvTuning t;
    t.waves = waves_opt;
    t.skinny_version = 2;
    t.trace = trace;
    t.trace_groups = trace_groups;
    return launch_skinny(g, packed, X, ldx, Y, ldy, batch, workspace, t, static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : 4;
}

}  // extern "C"
