/*
 * topk_attn_debug.h -- test and measurement aids of libtopk_attn, kept apart from the
 * method's boundary (topk_attn.h).  Nothing here is needed to run the decode path.
 */
#ifndef TOPK_ATTN_DEBUG_H
#define TOPK_ATTN_DEBUG_H

#include "topk_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Debug/measurement: write the full fp32 score matrix S = q K^T of `layer`
 * to scores [B, Hq, max_tokens] (device); entries beyond a sequence's length are
 * left untouched. */
int topk_attn_scores(topk_attn_t* h, int layer, const void* q, float* scores, void* hip_stream);

/* After the stream has been synchronised by the caller: number of (sequence, head)
 * pairs of the last decode whose filtered candidate list was unusable and were
 * recomputed by the full path.  Copies a few bytes device->host (synchronous). */
int topk_attn_last_fallbacks(topk_attn_t* h, int* n_heads);

/* Measurement aid: when enabled, every decode records a HIP event on its stream just
 * before and just after the key-scan kernel (up to 512 decodes between two reads).
 * Enabling creates the events (host resources only) and clears earlier records. */
int topk_attn_set_scan_timing(topk_attn_t* h, int enable);

/* After the caller has synchronised the stream: total milliseconds between the event
 * pairs recorded since the last read and the number of pairs; clears the records. */
int topk_attn_scan_time(topk_attn_t* h, double* total_ms, int* n_calls);

/* Measurement aid: stream `bytes` (multiple of 16) from `src` (device) with 128-bit
 * loads in the access shape of the key scan (16 KiB tiles per wave, sixteen loads in flight)
 * and write one checksum word per workgroup to `sink` (device, >= 64 KiB).
 * Gives the read-bandwidth ceiling the key scan is compared against. */
int topk_attn_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream);

/* Identifier of the sources the library was built from (a hash the build script passes in;
 * "unknown" for a build made otherwise).  Lets tests and recorded measurements tell a stale
 * binary from the sources beside it. */
const char* topk_attn_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* TOPK_ATTN_DEBUG_H */
