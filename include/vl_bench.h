/*
 * Measurement hooks for the benchmark.  NOT part of the library's boundary (include/vl.h):
 * nothing a user of the verifier needs, and nothing the tests of the method call.
 */
#ifndef VL_BENCH_H
#define VL_BENCH_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* libvlbench.so.  One launch that only reads `bytes` bytes (a multiple of 16, 16-byte aligned)
 * of buf [device] with 16-byte loads: what a plain streaming read reaches on the device, to
 * put beside the verifier's bytes per second.  sink [device]: one word, practically never
 * written.  stream: a hipStream_t.  Asynchronous.  Returns 0, -1 (a pointer missing),
 * -2 (length or alignment) or -6 (the launch failed). */
int32_t vl_stream_read_probe(const void *buf, uint64_t bytes, uint32_t *sink, void *stream);

/* libvl.so (it has to act inside a call of the library).  The next vl_verify_multi /
 * vl_verify_batch call on this thread records the two hipEvent_t (caller-owned, either may be
 * NULL) on its stream immediately before and after the candidate-walk kernel, the one that
 * reads the candidate rows.  One-shot. */
int32_t vl_verify_time_next(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif
