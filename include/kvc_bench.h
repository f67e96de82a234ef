/*
 * kvc_bench.h - measurement hooks of libkvc.  Not part of the product ABI: nothing a model
 * needs is declared here.  A benchmark uses them to time the launches inside
 * kvc_paged_decode with HIP events on the stream the kernels run on, and to measure the
 * streaming-read rate of the GPU it runs on, to set beside the kernels' rates.
 * Conventions as in kvc.h.  Host side these calls share one lock; they may be called from any
 * thread, but the recording covers the calls of the whole process.
 */
#ifndef KVC_BENCH_H_
#define KVC_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* kvc_profile_begin(n) makes the next n calls of kvc_paged_decode record HIP event pairs on
 * their stream around each of its three launches: the chunk kernel over the long items (it
 * streams nearly all of K and V), the same kernel over the short items, and the combine kernel;
 * n = 0 switches recording off and releases the events.  At most 4096 calls.              */
int kvc_profile_begin(int n);

/* Pauses (0) or resumes (non-zero) the recording without releasing anything, so that a
 * benchmark can time every k-th call only.                                              */
int kvc_profile_enable(int on);

/* Waits for the recorded events and writes up to `cap` durations in milliseconds to the host
 * arrays chunk_ms, short_ms and combine_ms (each may be NULL), returning the number of recorded
 * calls in *count (host).                                                               */
int kvc_profile_collect(float* chunk_ms, float* short_ms, float* combine_ms, int cap, int* count);

/* Bandwidth probe: reads `bytes` (a multiple of 16) of device memory at `src` once with 16-byte
 * non-temporal loads, grid-stride, and writes one 32-bit checksum per workgroup to `sink`
 * (device, at least `workgroups` words).                                                */
int kvc_stream_read_probe(const void* src, size_t bytes, uint32_t* sink, int workgroups,
                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVC_BENCH_H_ */
