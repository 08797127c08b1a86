/*
 * sip_diag.h -- measurement and diagnostic entry points of the MI355X batched token sampler.
 *
 * Nothing here is needed to sample: these calls time the library's kernels, measure what the
 * memory system gives a bare read in the streaming kernel's launch shape, and report launch
 * shapes.  They live in the same shared library as the entry points of sip.h.
 */
#ifndef SIP_DIAG_H_
#define SIP_DIAG_H_

#include "sip.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Profiling aid.  Arms a one-shot hook on the calling host thread: the next sampling call made
 * by this thread that takes the single-pass path launches its three kernels with the given
 * hipEvent_t handles (created by the caller with timing enabled) attached to the kernel
 * dispatches themselves: `stream_start` / `stream_stop` take the begin and end time stamps of
 * the streaming kernel -- the one pass over the logits, Sec. 5.1's dense row-wise work --,
 * `finish_*` those of the finishing kernel (one workgroup per row on the list the pass left) and
 * `rescue_*` those of the kernel behind it that takes the rows the list did not settle, so that a
 * caller reads each kernel's duration with hipEventElapsedTime without any extra packet between
 * them.  Any pointer may be NULL; all NULL disarms.  No effect on results.
 */
void sip_profile_kernel_events(void* stream_start, void* stream_stop, void* finish_start, void* finish_stop,
                               void* rescue_start, void* rescue_stop);

/*
 * Measurement aid: enqueue a bare streaming read of `bytes` bytes (a multiple of 16 is read) at
 * `src` (device, 16-byte aligned) in the launch shape of the streaming kernel -- `workgroups`
 * workgroups of 512 threads, each on one contiguous piece, 16-byte loads -- that only adds up
 * what it reads.  What this takes is what the memory system gives a kernel of that shape on
 * this machine: the figure the streaming kernel's time is set against beside the published
 * peak.  `workspace`: device, at least 4 * workgroups bytes (one partial sum per workgroup is
 * written).  start_event / stop_event: hipEvent_t handles that take the dispatch's own begin
 * and end time stamps, or NULL.
 */
sip_status sip_probe_read(const void* src, size_t bytes, int32_t workgroups, void* workspace,
                          size_t workspace_bytes, void* start_event, void* stop_event, void* hip_stream);

/*
 * Diagnostic, HOST only: into how many chunks (workgroups of the streaming kernel) a row of this
 * shape is cut; t_shards = 0 for logits in one matrix, else V = t_shards * V_shard.  0 = the shape
 * is served by the exact multi-pass kernel alone, -1 = invalid arguments.  A row's chunks are
 * whole units of 64 16-byte loads, dealt out evenly (to each vocabulary piece, if there are
 * pieces); none is empty.
 */
int32_t sip_plan_chunks(int32_t B, int32_t V, sip_dtype dtype, int32_t t_shards);

#ifdef __cplusplus
}
#endif
#endif /* SIP_DIAG_H_ */
