/*
 * topk_attn.h -- C ABI of the MI355X (gfx950) top-k attention decode library.
 *
 * The library implements one operator: the per-step "top-k attention" decode of
 * arXiv 2502.06766 (Methodology, "Top-k Attention: Accelerating Decoding", and
 * Algorithm 1 "Top-k KV Cache Decoding") in its exact-search form, with the whole
 * KV cache resident in GPU memory.  For every query head it
 *   1. scores the query against all N cached keys of its KV head with the raw dot
 *      product (the paper's search metric; S = q K^T of Eq. 1),
 *   2. finds the k largest scores `vals` and their positions `I`
 *      (Algorithm 1's  vals, I <- knn_search(q, K_index[l], k)),
 *   3. returns Softmax(vals / sqrt(head_dim)) . V[I]  (Algorithm 1's attention
 *      step over the retrieved rows).
 * With grouped-query attention, query head h reads KV head h / (n_q_heads /
 * n_kv_heads); every query head selects its own k positions.
 *
 * All pointers named "device" are GPU addresses on the configured device; the
 * library never allocates or frees device memory, never synchronises the device
 * in append/decode, and never touches host copies of the cache.  Calls on one
 * handle must not overlap in time (no internal locking).  Every function returns
 * a TOPK_ATTN_* code; argument errors are detected on the host before anything
 * is enqueued and leave the handle unchanged.
 */
#ifndef TOPK_ATTN_H
#define TOPK_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct topk_attn topk_attn_t; /* opaque, host memory owned by the library */

enum {
    TOPK_ATTN_OK = 0,
    TOPK_ATTN_EINVAL = 1,       /* null pointer, index out of range, k < 1, empty cache ... */
    TOPK_ATTN_ECAPACITY = 2,    /* append would exceed max_tokens */
    TOPK_ATTN_EUNSUPPORTED = 3, /* head_dim / dtype / head grouping the kernels do not cover */
    TOPK_ATTN_EDEVICE = 4,      /* a HIP call failed */
    TOPK_ATTN_ENOMEM = 5,       /* host allocation failed, or a caller buffer is too small */
    TOPK_ATTN_ESCRATCH = 6      /* topk_attn_decode_static: the configuration needs more per-call scratch
                                   than the library's built-in buffer holds */
};

enum { TOPK_ATTN_F32 = 0, TOPK_ATTN_F16 = 1, TOPK_ATTN_BF16 = 2 }; /* element type of q, K, V */

/* Which selection pipeline decode uses (see topk_attn_set_path). */
enum {
    TOPK_ATTN_PATH_AUTO = 0,    /* filtered scan when the shape allows it, else full */
    TOPK_ATTN_PATH_FULL = 1,    /* always materialise all N scores and radix-select over them */
    TOPK_ATTN_PATH_FILTER = 2,  /* sampled-threshold scan whenever its candidate list fits the
                                   workspace, also for short caches (heads whose candidate list
                                   under- or overflows are still redone exactly) */
    TOPK_ATTN_PATH_INDEX = 3,   /* approximate search over the int8 key index with exact refinement
                                   (needs index_kind = TOPK_ATTN_INDEX_INT8); where the filtered scan
                                   does not apply (short caches, dense k, several queries) the exact
                                   path runs instead */
    TOPK_ATTN_PATH_PAGES = 4    /* sub-linear search: the key scan skips the pages the coarse page index
                                   rules out (needs index_kind = TOPK_ATTN_INDEX_PAGES).  Exact: the
                                   selection of the plain scan (out may differ in the last bits: the
                                   partial sums are added in another order), unless
                                   topk_attn_set_page_bound_scale has shrunk the bound.  Where the filtered scan does not apply (short
                                   caches, dense k, several queries, head groups above 4) the exact path runs */
};

/* Search index kept beside the keys (Algorithm 1's build_index; the paper leaves the kind of
 * index open, from a plain list to approximate structures). */
enum {
    TOPK_ATTN_INDEX_NONE = 0,   /* the key array itself: exact search */
    TOPK_ATTN_INDEX_INT8 = 1,   /* plus a compressed copy of every key row: int8 codes
                                   rint(x * 127 / amax) and one fp32 scale amax / 127 per row
                                   (amax = largest magnitude of the row; rows below 2^-100 are coded
                                   as zero).  16-bit dtypes, head_dim 64, 128 or 256, Hq/Hkv <= 4. */
    TOPK_ATTN_INDEX_PAGES = 2   /* plus a coarse index over pages of 64 consecutive tokens (the paper's
                                   sub-linear retrieval; the kind of index is left open there): per page
                                   a centre c (mean of its keys, in the cache dtype) and two fp32 numbers,
                                   a radius r >= |k - c| for every key k of the page and |c|.  A page
                                   cannot hold a key that scores more than q . c + |q| r (Cauchy-Schwarz).
                                   16-bit dtypes, Hq/Hkv <= 4. */
};

typedef struct {
    uint32_t struct_size;   /* sizeof(topk_attn_config), for ABI versioning */
    int32_t n_layers;       /* L: independent caches, one per transformer layer */
    int32_t n_seqs;         /* B: sequences decoded together in one call */
    int32_t n_q_heads;      /* Hq */
    int32_t n_kv_heads;     /* Hkv, must divide Hq; Hq/Hkv <= 128 (<= 16 for fp32 caches) */
    int32_t head_dim;       /* d in {32, 64, 128, 256} */
    int64_t max_tokens;     /* capacity N_cap per (layer, sequence) */
    int32_t max_k;          /* largest k decode will be called with (<= 2^28); sizes the workspace */
    int32_t dtype;          /* TOPK_ATTN_F32 / F16 / BF16 for q, K and V alike */
    int32_t device;         /* HIP device ordinal */
    int32_t max_window;     /* largest `window` topk_attn_decode_window will be called with (0 if unused) */
    int32_t max_queries;    /* largest n_queries topk_attn_decode_multi will be called with (0 or 1 if
                               unused); the workspace grows in proportion */
    int32_t index_kind;     /* TOPK_ATTN_INDEX_*; the index lives in kv_storage after K and V */
    void* kv_storage;       /* device, >= topk_attn_kv_bytes(), 256-byte aligned, caller-owned */
    size_t kv_bytes;
    void* workspace;        /* device, >= topk_attn_workspace_bytes(), 256-byte aligned, caller-owned */
    size_t workspace_bytes;
} topk_attn_config;

/* Bytes of cache storage for the configuration: K then V, each laid out
 * [layer][seq][kv_head][max_tokens][head_dim] in `dtype` (2 L B Hkv N_cap d e bytes;
 * the paper's 2NDL cache of the Introduction with D = Hkv*d), each rounded up to 256 bytes.
 * With TOPK_ATTN_INDEX_INT8 the codes [layer][seq][kv_head][max_tokens][head_dim] int8 and
 * then the scales [layer][seq][kv_head][max_tokens] fp32 follow (each rounded up to 256
 * bytes).  With TOPK_ATTN_INDEX_PAGES the page centres [layer][seq][kv_head][P][head_dim] in
 * `dtype` and then [layer][seq][kv_head][P][2] fp32 (radius, centre norm) follow, P =
 * ceil(max_tokens / 64): 1.6 % of K at head_dim 128.  0 on invalid config. */
size_t topk_attn_kv_bytes(const topk_attn_config* cfg);

/* Bytes of scratch the kernels need (score buffer, candidate lists, partial sums,
 * per-sequence lengths).  0 on invalid config. */
size_t topk_attn_workspace_bytes(const topk_attn_config* cfg);

/* Build a handle over caller-owned storage (Algorithm 1's build_index for the exact
 * "list" index: the head-major key array itself is the index).  Zeroes the lengths
 * (synchronously).  The storage must stay valid until topk_attn_destroy. */
int topk_attn_create(const topk_attn_config* cfg, topk_attn_t** out);

/* Append n_new tokens to the cache of (layer, seq): Algorithm 1's concat of the new
 * k, v (and, with a large n_new, the bulk import of a prefilled cache).
 * k_new / v_new: device, element (t, h, c) at  base[t*token_stride + h*head_stride + c],
 * strides in elements (token-major [n_new, Hkv, d]: token_stride = Hkv*d, head_stride = d;
 * head-major [Hkv, n_new, d]: token_stride = d, head_stride = n_new*d).  Rows must be
 * 16-byte aligned.  The data is copied on `hip_stream` (a hipStream_t, may be NULL for
 * the default stream); the source may be reused once the stream has passed the call.
 * Errors: EINVAL (null, range, n_new < 0, misaligned), ECAPACITY. n_new == 0 is a no-op.
 * The handle keeps a host copy of every length (argument checks, launch shapes) that advances
 * once per call: an append recorded into a HIP graph must not be replayed (decode calls may). */
int topk_attn_append_kv(topk_attn_t* h, int layer, int seq, const void* k_new, const void* v_new,
                        int64_t n_new, int64_t token_stride, int64_t head_stride, void* hip_stream);

/* The per-step concat of Algorithm 1 for a whole batch: append n_new tokens to EVERY
 * sequence of `layer` in one call (two launches whatever B is, three with an int8 index;
 * topk_attn_append_kv costs one per sequence).  k_new / v_new: device [B, n_new, Hkv, d], contiguous, 16-byte
 * aligned.  Errors: EINVAL, ECAPACITY if any sequence would exceed max_tokens (nothing is
 * enqueued then).  n_new == 0 is a no-op. */
int topk_attn_append_step(topk_attn_t* h, int layer, const void* k_new, const void* v_new, int64_t n_new,
                          void* hip_stream);

/* One decode step of `layer` for all B sequences: steps 1-3 above over all tokens
 * currently cached for (layer, b).  k_eff = min(k, N_b).
 *   q     device [B, Hq, d] in the cache dtype
 *   out   device [B, Hq, d] fp32
 *   idx   device [B, Hq, k] int32 or NULL: selected positions, in no particular order;
 *         slots >= k_eff hold -1
 *   vals  device [B, Hq, k] fp32 or NULL: raw (unscaled) scores q.K[idx]; slots >= k_eff
 *         hold -inf
 *   lse   device [B, Hq] fp32 or NULL: log-sum-exp of vals/sqrt(d) over the selection
 *         (lets a caller merge with attention over further keys, e.g. a recent window)
 * Ties between equal scores go to the lower position.  Scores are accumulated in fp32.
 * Asynchronous on `hip_stream`.  Errors: EINVAL (null h/q/out, layer range, k < 1,
 * k > max_k, a sequence with no tokens), EDEVICE.
 * The launch shapes are chosen from the cached lengths at call time: a decode recorded into a
 * HIP graph may be replayed as long as no sequence of the layer has grown since. */
int topk_attn_decode(topk_attn_t* h, int layer, const void* q, int k, float* out, int32_t* idx,
                     float* vals, float* lse, void* hip_stream);

/* topk_attn_decode for callers that cannot allocate device memory for the call or hand over a
 * workspace they may reuse: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  Same arguments, same kernels and bit-identical results, but every per-call
 * buffer (sample scores, thresholds, candidate lists, the score buffer of the exact redo, partial
 * sums; internal idx / vals when the caller passes none) lives in a buffer built into the
 * library: a device array of TOPK_ATTN_STATIC_SCRATCH_BYTES that every GPU the library runs on
 * holds until the process ends.  Only the cache lengths are still read from the handle's
 * workspace.  The call allocates and frees nothing and enqueues kernels only.
 * Limit: ESCRATCH (nothing enqueued) if topk_attn_workspace_bytes(cfg) minus the lengths' share
 * (n_layers * n_seqs * 4, rounded up to 256) exceeds TOPK_ATTN_STATIC_SCRATCH_BYTES -- one
 * Llama-8B-shaped layer of 128k tokens at k = 2048 fits, a million-token layer does not.
 * All calls on one GPU, from whatever handle, share the one array: the call clears the words
 * that must start at zero itself, and two such calls that overlap in time on one GPU race. */
#define TOPK_ATTN_STATIC_SCRATCH_BYTES ((size_t)96 << 20)
int topk_attn_decode_static(topk_attn_t* h, int layer, const void* q, int k, float* out, int32_t* idx,
                            float* vals, float* lse, void* hip_stream);

/* Decode step with the recent-token window of Algorithm 1 (its K_gen / V_gen, which the
 * paper likens to windowed attention): for each sequence the last min(window, N_b) cached tokens are always
 * attended, the k-nearest-neighbour search runs over the older prefix only
 * (k_eff = min(k, N_b - window)), and one softmax spans the retrieved and the window scores
 * (the algorithm's window line is read as a joint softmax over both parts applied to
 * [V[I]; V_gen]).  idx / vals report the search result over the prefix; lse covers both parts.
 * window == 0 is topk_attn_decode.  Extra error: EINVAL if window < 0 or > max_window.
 * All work is enqueued on hip_stream. */
int topk_attn_decode_window(topk_attn_t* h, int layer, const void* q, int k, int window, float* out,
                            int32_t* idx, float* vals, float* lse, void* hip_stream);

/* Several queries per sequence against the cache in one pass over the keys (a chunk of M
 * consecutive queries, as in building the cache chunk by chunk -- the paper's suggestion to use top-k
 * attention when the cache is built, in the section on million-token cache generation -- or in
 * verifying drafted tokens): each of the M queries of a sequence gets its own exact
 * top-k search, softmax and weighted value sum, exactly as if topk_attn_decode_window had
 * been called once per query, but the keys are read once per block of up to 32
 * (query, head) rows of a KV head instead of once per query.
 *   q     device [B, M, Hq, d];  out [B, M, Hq, d];  idx / vals [B, M, Hq, k];  lse [B, M, Hq]
 *   causal != 0: the M queries are the last M cached tokens' queries, query m attends only
 *         to the first N_b - (M - 1 - m) tokens (its own token and everything before it);
 *         the window and k_eff are taken relative to that visible length.
 *   causal == 0: every query sees all N_b tokens.
 * n_queries == 1 is topk_attn_decode_window.  Extra errors: EINVAL if n_queries < 1,
 * n_queries > max(1, max_queries), or (causal) a sequence holds fewer than n_queries tokens. */
int topk_attn_decode_multi(topk_attn_t* h, int layer, const void* q, int n_queries, int causal, int k,
                           int window, float* out, int32_t* idx, float* vals, float* lse,
                           void* hip_stream);

/* Host-only helper for the paper's layer-wise settings of k ("Layer-Wise Settings for k":
 * a fixed total budget sum_l k_l, spent either uniformly or increasing linearly from the
 * first to the last layer).  Writes k_out[0 .. n_layers) with sum exactly total_k and
 * k_l proportional (before rounding) to 1 + (last_over_first - 1) * l / (n_layers - 1);
 * last_over_first == 1 gives the uniform split.  Rounding: floor, then the remainder goes
 * one each to the layers with the largest fractional parts (later layer first on ties).
 * Errors: EINVAL if k_out is NULL, n_layers < 1, total_k < n_layers (every layer needs
 * k >= 1), last_over_first <= 0 or not finite, or a k_l would not fit in int32. */
int topk_attn_k_schedule(int64_t total_k, int n_layers, double last_over_first, int32_t* k_out);

/* Decode steps of n_layers consecutive layers [layer0, layer0 + n_layers) with a per-layer k
 * (e.g. from topk_attn_k_schedule), enqueued back to back on `hip_stream`: the same work as
 * n_layers calls of topk_attn_decode_window, one per layer, each with its own query block.
 * (In a transformer layer l+1's query depends on layer l's output; this entry point serves
 * callers that have all queries at hand, such as replaying recorded queries or measuring
 * a whole-model decode step.)
 *   q     device [n_layers, B, Hq, d];  out device [n_layers, B, Hq, d] fp32
 *   k     host   [n_layers] int32, each in [1, max_k]
 *   idx / vals  device or NULL: ragged concatenation, layer l's [B, Hq, k[l]] block starts
 *         at element B * Hq * (k[0] + ... + k[l-1])
 *   lse   device [n_layers, B, Hq] or NULL
 * Errors as topk_attn_decode_window for any layer; nothing is enqueued unless all layers
 * pass the checks. */
int topk_attn_decode_layers(topk_attn_t* h, int layer0, int n_layers, const void* q, const int32_t* k,
                            int window, float* out, int32_t* idx, float* vals, float* lse,
                            void* hip_stream);

/* Scale beta in (0, 1] of the page radius in the bound q . c + beta |q| r that decides which pages the
 * key scan of TOPK_ATTN_PATH_PAGES reads.  1 (the default) is exact.  Below 1 fewer pages are read and a
 * key whose page was skipped is missed even if its score belongs to the k largest: approximate search,
 * recall@k against the exact path is the figure of merit; what is returned carries exact scores.
 * EINVAL without a page index or for beta outside (0, 1]. */
int topk_attn_set_page_bound_scale(topk_attn_t* h, float beta);

/* Tokens currently cached for (layer, seq); -1 on bad arguments. */
int64_t topk_attn_length(const topk_attn_t* h, int layer, int seq);

/* Forget the tokens of (layer, seq) (length := 0); enqueued on hip_stream. */
int topk_attn_reset(topk_attn_t* h, int layer, int seq, void* hip_stream);

/* Choose the search (TOPK_ATTN_PATH_*); default AUTO, the exact search.  TOPK_ATTN_PATH_INDEX is
 * the method's approximate search over the int8 index; FULL and FILTER only force one of the two
 * exact pipelines AUTO chooses between (same results; tests use them).  EINVAL for an unknown
 * value, or TOPK_ATTN_PATH_INDEX on a handle without an index.  With TOPK_ATTN_PATH_INDEX
 * the result of decode is approximate: a key whose coded score falls below the candidate
 * threshold is missed even if its exact score belongs to the k largest (recall@k against
 * the exact path is the figure of merit); positions returned always carry their exact
 * scores, and the softmax runs over exactly those.  topk_attn_scores then dumps the
 * approximate scores  float(codes(q) . codes(K_i)) * (scale_q * scale_i). */
int topk_attn_set_path(topk_attn_t* h, int path);

const char* topk_attn_strerror(int code);

/* Frees the host handle only. */
int topk_attn_destroy(topk_attn_t* h);

#ifdef __cplusplus
}
#endif
#endif /* TOPK_ATTN_H */
