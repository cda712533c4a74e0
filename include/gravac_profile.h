/*
 * gravac_profile.h - measurement aid of the MI355X gradient-compression library: gravac_compress with the
 * caller's HIP events recorded around the call and around its pass over the gradient.  Not part of the
 * compression path (gravac.h); benchmarks use it to time the dominant kernel on the stream it runs on.
 */
#ifndef GRAVAC_PROFILE_H
#define GRAVAC_PROFILE_H

#include "gravac.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Four events of the caller (hipEvent_t, created with timing enabled, passed as void*), all four required.
 * The library records them on the call's stream and keeps nothing: after the stream has been synchronised,
 * hipEventElapsedTime(pass_begin, pass_end) is the duration of the streaming kernel (error feedback, Sec. III-B,
 * fused with the collection of the Top-k candidates, Sec. II-C) and hipEventElapsedTime(call_begin, call_end)
 * that of the whole call, first to last kernel.
 */
typedef struct gravac_profile_events {
    void* call_begin; /* recorded before the first kernel */
    void* pass_begin; /* the streaming kernel's own begin time stamp */
    void* pass_end;   /* ... and its end time stamp */
    void* call_end;   /* recorded after the last kernel */
} gravac_profile_events;

/*
 * gravac_compress (same arguments, same results) with `events` recorded as described above.  Returns
 * GRAVAC_ERR_CAPTURE on a stream that is being captured into a graph (a replay would record the events again),
 * GRAVAC_ERR_INVALID_ARG if `events` or one of its members is NULL.
 */
int gravac_compress_profiled(const float* grad, float* residual, int64_t n,
                             const double* cf_list, int n_cf, int commit,
                             const int64_t* seg_offsets, int n_seg,
                             int32_t* out_idx, float* out_val, int64_t out_capacity,
                             int64_t* out_count, double* out_stats,
                             void* workspace, size_t workspace_bytes,
                             unsigned flags, void* stream, const gravac_profile_events* events);

#ifdef __cplusplus
}
#endif
#endif /* GRAVAC_PROFILE_H */
