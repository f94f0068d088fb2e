/*
 * flashblock_prof.h - measurement hooks of libflashblock.so.  Not part of the product interface
 * (include/flashblock.h): the two calls below are what a benchmark needs to time the streaming
 * attention kernel of a call by itself, with HIP events recorded on the call's own stream
 * between the kernels the call launches.  Everything else about them (arguments, results,
 * errors) is as for the plain entry point each one wraps.
 */
#ifndef FLASHBLOCK_PROF_H_
#define FLASHBLOCK_PROF_H_

#include "flashblock.h"

#ifdef __cplusplus
extern "C" {
#endif

/* fb_external_partial_ex that also fills three caller-created HIP events (hipEvent_t cast to void*,
 * created with timing enabled) on hip_stream.  For bf16 shapes ev_begin and ev_attn_end are the
 * streaming attention kernel's own start and stop events (the launch carries them: they hold the
 * timestamps of the kernel's dispatch, the duration a profiler's kernel trace reports); for fp32
 * shapes they are recorded immediately before and after that launch.  ev_end is recorded after the
 * split combine.  Any of the three may be NULL.  Results are identical to fb_external_partial_ex. */
fb_status fb_external_partial_prof(const fb_shape* shape, const void* q, const void* k_prefix,
                                   const void* v_prefix, float* o_part, float* m_part,
                                   float* lse_part, int32_t n_splits, void* workspace,
                                   size_t workspace_bytes, void* ev_begin, void* ev_attn_end,
                                   void* ev_end, void* hip_stream);

/* fb_refresh_step that also records three caller-created HIP events, as
 * fb_external_partial_prof does (before the streaming kernel, between it and the combine, after
 * the combine).  Any of the three may be NULL.  Results are identical to fb_refresh_step. */
fb_status fb_refresh_step_prof(const fb_shape* shape, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_block, const void* v_block,
                               float* o_part, float* m_part, float* lse_part, void* out,
                               float* lse_out, void* workspace, size_t workspace_bytes,
                               void* ev_begin, void* ev_attn_end, void* ev_end, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHBLOCK_PROF_H_ */
