/*
 * libmoqae -- measurement aids.  NOT part of the method and not needed by any caller of moqae.h: these entry
 * points exist so that a benchmark can time the library's dominant kernel alone, as a profiler does, and can
 * measure the read bandwidth a plain streaming kernel reaches on the same GPU (the practical ceiling that
 * the decode kernel's fraction of the HBM peak should be read against).
 */
#ifndef MOQAE_BENCH_H
#define MOQAE_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The decode calls this host thread makes from now on record the two given events (hipEvent_t passed as
 * void*, owned by the caller, created with timing enabled) on the call's stream right before and right
 * after the main kernel of the decode call.  Pass NULL, NULL to stop.  Returns MOQAE_OK.
 */
int moqae_bench_time_decode_kernel(void *event_begin, void *event_end);

/*
 * Read-only streaming kernel: reads `bytes` bytes (a multiple of 16; device pointer `buf`, 16-byte aligned)
 * once, with 16-byte loads issued back to back, folds them with XOR and leaves one word per workgroup in
 * `sink` (device, at least 4 * moqae_bench_stream_sink_words() bytes).  Enqueued on `stream`; returns
 * MOQAE_OK, MOQAE_E_INVAL or MOQAE_E_HIP.
 */
int moqae_bench_stream_read(const void *buf, uint64_t bytes, uint32_t *sink, void *stream);
uint32_t moqae_bench_stream_sink_words(void);

#ifdef __cplusplus
}
#endif
#endif /* MOQAE_BENCH_H */
