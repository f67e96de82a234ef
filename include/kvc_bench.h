/*
 * kvc_bench.h - measurement hooks of libkvc.  Not part of the product ABI: nothing a model
 * needs is declared here.  A benchmark uses them to time the launches inside
 * kvc_paged_decode with HIP events on the stream the kernels run on, and to measure the
 * streaming-read rate of the GPU it runs on, alone and with the decode's share of writes, to set
 * beside the kernels' rates.
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

/* A read stream shaped like the decode's, with its share of writes if asked for: `bytes` of device
 * memory at `src` (16-byte aligned) are read in items of item_bytes (a multiple of 512, at least
 * 4096), one workgroup per item at a time, and with adds != 0 every item is followed by one
 * hardware float add per 512 bytes read, into dst[item * (item_bytes / 512) ...] (device; at least
 * (bytes / item_bytes) * (item_bytes / 512) floats, else KVC_ERR_ARG): what the metric of 16-bit
 * rows of d = 128 asks for.  What is left of `bytes` after the last whole item is not read.  One
 * 32-bit checksum per workgroup goes to `sink` (device, at least `workgroups` words).    */
int kvc_stream_read_add_probe(const void* src, size_t bytes, size_t item_bytes, int adds, float* dst,
                              size_t dst_floats, uint32_t* sink, int workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVC_BENCH_H_ */
