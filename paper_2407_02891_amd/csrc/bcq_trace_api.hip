// Entry points of the tracing build of the GEMV (libbcq_trace.so; built by build.py --trace from
// bcq_gemv.hip compiled with -DBCQ_TRACE, bcq_pack.hip and this file; used by trace_gemv.py).  A
// diagnostic, not part of the product library: same kernel, plus time stamps per wave.
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

}  // extern "C"
