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
 * pairs of the last decode whose filtered candidate list turned out unusable (a segment
 * overflowed, or fewer than k keys reached the sampled threshold) and were recomputed
 * exactly.  Heads of sequences that cannot be filtered at all (a few tokens only, or k too
 * dense) are recomputed the same way by design and are not counted.  Copies a few bytes
 * device->host (synchronous). */
int topk_attn_last_fallbacks(topk_attn_t* h, int* n_heads);

/* After the caller has synchronised the stream: how many pages (64 tokens of one KV head) the key scan
 * of the last decode read, and how many the layer's caches hold.  Equal unless the decode went through
 * TOPK_ATTN_PATH_PAGES.  Copies the page mask device->host (synchronous). */
int topk_attn_last_pages_read(topk_attn_t* h, int64_t* pages_read, int64_t* pages_total);

/* After the caller has synchronised the stream: what the selection of the last decode found for each
 * (sequence, query, head) row that took the filtered path with the chip-wide selection: records[4 i + 0] = 0 if
 * the head's candidate list was used or its keys were sorted again, 1 if it was selected from its full
 * score row, 2 if there was nothing to search, with the head's flag word in bits 8 and up (bit 8: its
 * sequence cannot be filtered, bit 9: the keys sorted again did not fit either, bit 10: forced redo); [4 i + 1] = keys
 * selected for certain (score bins above the one the k-th score falls in); [4 i + 2] = keys still to pick
 * from that bin; [4 i + 3] = candidates in that bin.  `records` is a host array of 4 * n_seqs * n_q_heads
 * words, times the queries per sequence of that decode.  TOPK_ATTN_EINVAL if the last decode took another path.  Copies device->host (synchronous). */
int topk_attn_last_selection_records(topk_attn_t* h, uint32_t* records);

/* After the caller has synchronised the stream: copies the first `bytes` bytes of one of the per-call arrays of
 * the handle's workspace to the host array `dst` (for tests that look at what a decode left behind).  Names:
 * "thr", "bins", "samp", "seg_cnt", "seg_max", "seg_cnt2", "flags", "tailrec", "page_mask", "page_cnt",
 * "page_list", "hist", "cand", "bnd".  EINVAL for another name or more bytes than the array holds.  The second call
 * reports dims[0..5] = entries per candidate list, entries per boundary list, scan workgroups the per-bin counts
 * have room for, most wave segments per head, and the wave segments and entries per segment of the last
 * filtered decode (0, 0 if the last decode was not filtered). */
int topk_attn_debug_read_workspace(topk_attn_t* h, const char* name, void* dst, size_t bytes);
int topk_attn_debug_read_workspace_dims(topk_attn_t* h, int32_t* dims);

/* Measurement aid for the worst case of the filtered path: when enabled, every head of a decode
 * that takes the filtered path is treated like a head whose candidate list turned out unusable
 * (nothing passes its scan; all its keys are rescored exactly and selected from the full score
 * row).  Results are unchanged; such heads are not counted by topk_attn_last_fallbacks, which
 * counts lists that should have been usable. */
int topk_attn_debug_force_redo(topk_attn_t* h, int enable);

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
