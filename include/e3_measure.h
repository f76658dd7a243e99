/*
 * libe3 -- measurement hooks.  NOT part of the library's interface: these two entry
 * points exist so that a benchmark can time the library's own dispatches and compare
 * them with a plain read of the same memory.  They perform none of the method's
 * arithmetic, may change or disappear, and a product caller has no use for them.
 * Conventions (device pointers, stream, return codes) as in e3.h.
 */
#ifndef E3_MEASURE_H
#define E3_MEASURE_H

#include "e3.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The next e3_sample_entropy / e3_logprob_entropy(_gap) / e3_read_probe
 * call made by this host thread attaches the two events (hipEvent_t created by the caller with timing
 * enabled; either may be NULL) to its vocabulary-pass dispatch: `start_event` then holds
 * the time the kernel began to execute and `stop_event` the time it ended (when the call
 * launches more than one kernel -- a small batch with a workspace, a training-side call that
 * also returns the batch sums -- begin of the first kernel and end of the last),
 * so hipEventElapsedTime gives the kernel's own duration without the cost of marker
 * packets recorded around it.  The hook is consumed by the first such call that reaches its
 * launch (a call rejected by its argument checks, or with rows == 0, leaves it in place);
 * calling it again before replaces the events; NULL, NULL clears it.  Always returns E3_OK.
 */
int e3_time_next_launch(void* start_event, void* stop_event);

/*
 * Diagnostic, for callers that measure: read `bytes` bytes of device memory once, with
 * the access pattern of the vocabulary pass (16-byte non-temporal loads, eight-wave
 * workgroups streaming contiguous 16-KiB runs), and write E3_READ_PROBE_SUMS xor
 * checksums (one per workgroup, unused slots zero; their xor is the xor of all 32-bit
 * words of the buffer) to sums_out [E3_READ_PROBE_SUMS] uint32, device.  It performs none
 * of the method's arithmetic: timing it on the same buffers gives the read rate that the
 * kernels' achieved GB/s can be compared with (meant for buffers of a hundred MB and more;
 * small buffers get few workgroups).  bytes must be a multiple of 16 (E3_ERR_SHAPE) and
 * buf 16-byte aligned (E3_ERR_ALIGN); bytes == 0 writes zeros.
 */
#define E3_READ_PROBE_SUMS 2048
int e3_read_probe(const void* buf, int64_t bytes, uint32_t* sums_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* E3_MEASURE_H */
