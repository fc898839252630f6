// Host side of libtopk_attn: handle, argument checks, workspace layout, launches.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "../../include/topk_attn.h"
#include "../../include/topk_attn_debug.h"
#include "device_utils.h"
#include "internal.h"

using namespace tka;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int elem_bytes(int dtype) { return dtype == TOPK_ATTN_F32 ? 4 : 2; }

struct WsLayout {
    size_t len, thr, bins, samp, seg_cnt, seg_max, seg_cnt2, flags, hmax, fallback, tailrec, qscale, q8, page_mask, page_cnt, page_list, hist, cand, bnd, scores, sel_idx, sel_val, part_acc, part_l, part_m, total;
    int cand_cap, bnd_cap, n_chunk_cap, hist_cap, page_words;
};

bool config_ok(const topk_attn_config* c, int* why) {
    *why = TOPK_ATTN_EINVAL;
    if (!c || c->struct_size != sizeof(topk_attn_config)) return false;
    if (c->n_layers < 1 || c->n_seqs < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return false;
    if (c->max_tokens < 1 || c->max_k < 1 || c->device < 0 || c->max_window < 0) return false;
    if (c->max_queries < 0 || c->max_queries > 4096) return false;
    if (c->index_kind != TOPK_ATTN_INDEX_NONE && c->index_kind != TOPK_ATTN_INDEX_INT8 &&
        c->index_kind != TOPK_ATTN_INDEX_PAGES)
        return false;
    if ((int64_t)c->n_seqs * (c->max_queries > 1 ? c->max_queries : 1) > 65535) return false;   // a grid dimension
    if (c->max_tokens > (int64_t)0x7FFFFF00) return false;   // positions are int32
    if (c->max_k > (1 << 28)) return false;                  // the candidate list (about 4 max_k entries) is indexed by int32
    if (c->n_seqs > 65535 || c->n_kv_heads > 65535) return false;
    *why = TOPK_ATTN_EUNSUPPORTED;
    if (c->dtype != TOPK_ATTN_F32 && c->dtype != TOPK_ATTN_F16 && c->dtype != TOPK_ATTN_BF16) return false;
    if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128 && c->head_dim != 256) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    if (c->n_q_heads / c->n_kv_heads > 128) return false;
    if (c->dtype == TOPK_ATTN_F32 && c->n_q_heads / c->n_kv_heads > 16) return false;   // plain-FMA scorer
    if (c->index_kind == TOPK_ATTN_INDEX_INT8 &&
        !index8_supported(c->dtype, c->head_dim, c->n_q_heads / c->n_kv_heads))
        return false;
    if (c->index_kind == TOPK_ATTN_INDEX_PAGES &&
        !pages_supported(c->dtype, c->head_dim, c->n_q_heads / c->n_kv_heads))
        return false;
    *why = TOPK_ATTN_OK;
    return true;
}

size_t kv_half_bytes(const topk_attn_config* c) {
    return align_up((size_t)c->n_layers * c->n_seqs * c->n_kv_heads * (size_t)c->max_tokens * c->head_dim *
                    elem_bytes(c->dtype));
}

// int8 index behind K and V: codes, then scales
size_t index_codes_bytes(const topk_attn_config* c) {
    if (c->index_kind != TOPK_ATTN_INDEX_INT8) return 0;
    return align_up((size_t)c->n_layers * c->n_seqs * c->n_kv_heads * (size_t)c->max_tokens * c->head_dim);
}
size_t index_scales_bytes(const topk_attn_config* c) {
    if (c->index_kind != TOPK_ATTN_INDEX_INT8) return 0;
    return align_up((size_t)c->n_layers * c->n_seqs * c->n_kv_heads * (size_t)c->max_tokens * sizeof(float));
}
// page index behind K and V: centres, then (radius, centre norm) pairs
int64_t page_cap_of(const topk_attn_config* c) { return (c->max_tokens + 63) / 64; }
size_t page_centres_bytes(const topk_attn_config* c) {
    if (c->index_kind != TOPK_ATTN_INDEX_PAGES) return 0;
    return align_up((size_t)c->n_layers * c->n_seqs * c->n_kv_heads * (size_t)page_cap_of(c) * c->head_dim * elem_bytes(c->dtype));
}
size_t page_balls_bytes(const topk_attn_config* c) {
    if (c->index_kind != TOPK_ATTN_INDEX_PAGES) return 0;
    return align_up((size_t)c->n_layers * c->n_seqs * c->n_kv_heads * (size_t)page_cap_of(c) * 2 * sizeof(float));
}
size_t kv_total_bytes(const topk_attn_config* c) {
    return 2 * kv_half_bytes(c) + index_codes_bytes(c) + index_scales_bytes(c) + page_centres_bytes(c) + page_balls_bytes(c);
}

WsLayout ws_layout(const topk_attn_config* c) {
    WsLayout w;
    const size_t BH = (size_t)c->n_seqs * (c->max_queries > 1 ? c->max_queries : 1) * c->n_q_heads;
    const int64_t max_k = c->max_k < c->max_tokens ? c->max_k : c->max_tokens;
    // candidate list per head.  A call with few KV-head streams splits each stream into many wave
    // segments (up to about 1024 waves over the chip, doubled where the split is rounded up).
    int64_t seg_max = 8 * ((512 + (int64_t)c->n_seqs * c->n_kv_heads - 1) / ((int64_t)c->n_seqs * c->n_kv_heads));
    if (seg_max > kMaxSeg) seg_max = kMaxSeg;
    // The boundary list takes the expected candidates (about 2 k at most) and a few dozen spare entries
    // per segment.  The segments of the candidate list are sized for keys whose scores come in runs
    // along the sequence (a passage the query attends to): a whole 64-key tile of candidates lands in
    // one segment at a time, so a segment that expects m such tiles gets room for m + 5 sqrt(m) + 4.
    w.bnd_cap = (int)(4 * max_k + 16384 + 48 * seg_max);
    {
        const Plan top = make_plan(c->max_tokens, (int)max_k);
        const double m = (double)top.c_hi / (64.0 * (double)seg_max);
        const int64_t lumpy = (int64_t)((double)seg_max * 64.0 * (m + 5.0 * sqrt(m) + 4.0));
        w.cand_cap = (int)(lumpy > w.bnd_cap ? lumpy : w.bnd_cap);
        // whole 128-byte lines per head and whole runs of kCandChunk per segment, however the list is split
        w.cand_cap = (int)(((int64_t)w.cand_cap + kMaxSeg * kCandChunk - 1) / (kMaxSeg * kCandChunk) * (kMaxSeg * kCandChunk));
    }
    const int64_t max_w = c->max_window < c->max_tokens ? c->max_window : c->max_tokens;
    w.hist_cap = (int)(seg_max / 4);            // scan workgroups per head (four wave segments each)
    // partial sums per head: the tail of the filtered path makes up to one per 128 selected rows, at least one per
    // four scan workgroups (and never more than scan workgroups fed the head), the gather one per 256; the window
    // adds one per 256 tokens
    {
        const int64_t by_k = ((int64_t)c->max_k + 127) / 128, by_wg = (w.hist_cap + 3) / 4;
        w.n_chunk_cap = (int)((by_k > by_wg ? by_k : by_wg) + (max_w + kGatherRows - 1) / kGatherRows);
    }
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    w.len = take((size_t)c->n_layers * c->n_seqs * sizeof(int32_t));
    w.thr = take(BH * sizeof(float));
    w.bins = take(BH * 2 * sizeof(float));
    w.samp = take(BH * kSampMax * sizeof(float));
    w.seg_cnt = take(BH * kMaxSeg * sizeof(uint32_t));
    w.seg_max = take(BH * kMaxSeg * sizeof(float));
    w.seg_cnt2 = take(BH * kMaxSeg * sizeof(uint32_t));
    w.flags = take(BH * sizeof(uint32_t));
    w.hmax = take(BH * sizeof(float));
    w.fallback = take(sizeof(uint32_t));
    w.tailrec = take(BH * 4 * sizeof(uint32_t));
    w.qscale = take(BH * sizeof(float));
    w.q8 = take(BH * (size_t)c->head_dim);
    w.page_words = (int)((page_cap_of(c) + 63) / 64);
    const size_t page_streams = c->index_kind == TOPK_ATTN_INDEX_PAGES ? (size_t)c->n_seqs * c->n_kv_heads : 0;
    w.page_mask = take(page_streams * (size_t)w.page_words * sizeof(uint64_t));
    w.page_cnt = take(page_streams * sizeof(uint32_t));
    w.page_list = take(page_streams * (size_t)w.page_words * 64 * sizeof(int32_t));
    w.hist = take(BH * (size_t)w.hist_cap * kTailBins * sizeof(uint32_t));
    w.cand = take(BH * (size_t)w.cand_cap * sizeof(uint64_t));
    w.bnd = take(BH * (size_t)w.bnd_cap * sizeof(uint64_t));
    w.scores = take(BH * (size_t)c->max_tokens * sizeof(float));
    w.sel_idx = take(BH * (size_t)c->max_k * sizeof(int32_t));   // stride is the requested k, up to max_k
    w.sel_val = take(BH * (size_t)c->max_k * sizeof(float));
    w.part_acc = take(BH * (size_t)w.n_chunk_cap * c->head_dim * sizeof(float));
    w.part_l = take(BH * (size_t)w.n_chunk_cap * sizeof(float));
    w.part_m = take(BH * (size_t)w.n_chunk_cap * sizeof(float));
    w.total = o;
    return w;
}

__global__ void append_kernel(const char* __restrict__ ksrc, const char* __restrict__ vsrc, char* __restrict__ kdst,
                              char* __restrict__ vdst, int64_t n_new, int Hkv, int chunks_per_row,
                              int64_t token_stride_b, int64_t head_stride_b, int64_t dst_head_stride_b,
                              int32_t* len_slot, int32_t new_len) {
    const int64_t total = n_new * Hkv * chunks_per_row;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % chunks_per_row);
        const int64_t th = i / chunks_per_row;
        const int h = (int)(th % Hkv);
        const int64_t t = th / Hkv;
        const int64_t so = t * token_stride_b + h * head_stride_b + (int64_t)c * 16;
        const int64_t d_o = h * dst_head_stride_b + (t * chunks_per_row + c) * 16;
        *reinterpret_cast<u32x4*>(kdst + d_o) = *reinterpret_cast<const u32x4*>(ksrc + so);
        *reinterpret_cast<u32x4*>(vdst + d_o) = *reinterpret_cast<const u32x4*>(vsrc + so);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *len_slot = new_len;
}

__global__ void set_len_kernel(int32_t* len_slot, int32_t v) { *len_slot = v; }

// n_new tokens for every sequence of a layer: source [B][n_new][Hkv][row], destination row
// len[b] + t of (b, h).  The lengths are bumped by a second kernel once every block has read them.
__global__ void append_step_kernel(const char* __restrict__ ksrc, const char* __restrict__ vsrc, char* __restrict__ kdst,
                                   char* __restrict__ vdst, const int32_t* __restrict__ len, int64_t total, int64_t n_new,
                                   int Hkv, int chunks_per_row, int64_t head_b) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % chunks_per_row);
        const int64_t th = i / chunks_per_row;
        const int h = (int)(th % Hkv);
        const int64_t bt = th / Hkv;
        const int64_t t = bt % n_new, b = bt / n_new;
        const int64_t d_o = (b * Hkv + h) * head_b + (((int64_t)len[b] + t) * chunks_per_row + c) * 16;
        *reinterpret_cast<u32x4*>(kdst + d_o) = *reinterpret_cast<const u32x4*>(ksrc + i * 16);
        *reinterpret_cast<u32x4*>(vdst + d_o) = *reinterpret_cast<const u32x4*>(vsrc + i * 16);
    }
}
// The same for a step small enough for one workgroup (a token or a few per sequence, no index to extend): the
// workgroup bumps the lengths itself once all its threads have placed their pieces, one launch instead of two.
constexpr int kAppendSmallThreads = 1024;
constexpr int64_t kAppendSmallPieces = 4 * kAppendSmallThreads;       // 16-byte pieces of K (and of V) per call: 256 rows of 256 bytes
__global__ void __launch_bounds__(kAppendSmallThreads)
append_step_small_kernel(const char* __restrict__ ksrc, const char* __restrict__ vsrc, char* __restrict__ kdst,
                         char* __restrict__ vdst, int32_t* len, int64_t total, int64_t n_new, int Hkv, int chunks_per_row,
                         int64_t head_b, int B) {
    for (int64_t i = threadIdx.x; i < total; i += kAppendSmallThreads) {
        const int c = (int)(i % chunks_per_row);
        const int64_t th = i / chunks_per_row;
        const int h = (int)(th % Hkv);
        const int64_t bt = th / Hkv;
        const int64_t t = bt % n_new, b = bt / n_new;
        const int64_t d_o = (b * Hkv + h) * head_b + (((int64_t)len[b] + t) * chunks_per_row + c) * 16;
        *reinterpret_cast<u32x4*>(kdst + d_o) = *reinterpret_cast<const u32x4*>(ksrc + i * 16);
        *reinterpret_cast<u32x4*>(vdst + d_o) = *reinterpret_cast<const u32x4*>(vsrc + i * 16);
    }
    __syncthreads();            // every thread has used the lengths it needed
    for (int b = threadIdx.x; b < B; b += kAppendSmallThreads) len[b] += (int32_t)n_new;
}
__global__ void bump_len_kernel(int32_t* len, int B, int32_t n_new) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) len[b] += n_new;
}

// Streaming read of n_vec 16-byte vectors: every wave walks 16 KiB tiles (16 independent
// 1 KiB-per-instruction loads in flight), the access shape of the key scan without its work.
__global__ void __launch_bounds__(256) read_probe_kernel(const u32x4* __restrict__ src, size_t n_vec, uint32_t* sink) {
    uint32_t acc = 0;
    const size_t lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (size_t)gridDim.x * 4;
    const size_t n_tiles = n_vec / 1024;
    for (size_t t = wave; t < n_tiles; t += n_waves) {
        const u32x4* p = src + t * 1024 + lane;
        u32x4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = p[u * 64];
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (size_t i = n_tiles * 1024 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec;
         i += (size_t)gridDim.x * blockDim.x) {
        const u32x4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x & 16383], acc);
}

__global__ void zero_words_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

}  // namespace

// Built-in scratch of topk_attn_decode_static: the per-call buffers of one decode (everything the
// handle's workspace holds except the cache lengths) for callers that bring no workspace of
// their own to that call.  One copy per GPU, at its own address, held until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)96 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on each GPU (the array's name is only a host-side stand-in for
// it), looked up once per device with that device current.
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;
static int scratch_address(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return TOPK_ATTN_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TOPK_ATTN_EDEVICE;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return TOPK_ATTN_OK;
}

constexpr int kTimingSlots = 512;

struct topk_attn {
    topk_attn_config cfg;
    WsLayout ws;
    size_t kv_half;
    std::vector<int64_t> len;   // host mirror of the device lengths, [L][B]
    int path;
    bool last_fast;
    bool last_static;           // the last decode used the built-in scratch
    bool force_redo;            // measurement aid, see topk_attn_debug_force_redo
    float page_beta;            // scale of the page radius in the page bound (1 = exact)
    bool last_paged;            // the last decode went through the page index
    bool last_tail;             // the last decode used the chip-wide selection (its per-head records are in the workspace)
    int last_queries;           // queries per sequence of the last decode
    int last_n_seg, last_seg_cap;   // the split of the last filtered decode's candidate lists (0: not filtered)
    int last_layer;
    char* scratch_dev;          // this device's copy of the built-in scratch
    int n_cu;                   // compute units of the device
    // optional event pairs around the key scan of each decode (measurement only)
    bool timing;
    std::vector<hipEvent_t> ev;  // 2 * kTimingSlots once enabled
    int ev_used;
};

extern "C" {

size_t topk_attn_kv_bytes(const topk_attn_config* cfg) {
    int why;
    if (!config_ok(cfg, &why)) return 0;
    return kv_total_bytes(cfg);
}

size_t topk_attn_workspace_bytes(const topk_attn_config* cfg) {
    int why;
    if (!config_ok(cfg, &why)) return 0;
    return ws_layout(cfg).total;
}

int topk_attn_create(const topk_attn_config* cfg, topk_attn_t** out) {
    if (!out) return TOPK_ATTN_EINVAL;
    *out = nullptr;
    int why;
    if (!config_ok(cfg, &why)) return why;
    if (!cfg->kv_storage || !cfg->workspace) return TOPK_ATTN_EINVAL;
    if (((uintptr_t)cfg->kv_storage | (uintptr_t)cfg->workspace) & (kAlign - 1)) return TOPK_ATTN_EINVAL;
    WsLayout w = ws_layout(cfg);
    if (cfg->kv_bytes < kv_total_bytes(cfg) || cfg->workspace_bytes < w.total) return TOPK_ATTN_ENOMEM;
    topk_attn* h = new (std::nothrow) topk_attn;
    if (!h) return TOPK_ATTN_ENOMEM;
    h->cfg = *cfg;
    h->ws = w;
    h->kv_half = kv_half_bytes(cfg);
    h->len.assign((size_t)cfg->n_layers * cfg->n_seqs, 0);
    h->path = TOPK_ATTN_PATH_AUTO;
    h->last_fast = false;
    h->timing = false;
    h->ev_used = 0;
    if (hipSetDevice(cfg->device) != hipSuccess) { delete h; return TOPK_ATTN_EDEVICE; }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess) { delete h; return TOPK_ATTN_EDEVICE; }
    h->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    h->last_static = false;
    h->force_redo = false;
    h->page_beta = 1.0f;
    h->last_paged = false;
    h->last_tail = false;
    h->last_queries = 1;
    h->last_n_seg = h->last_seg_cap = 0;
    h->last_layer = 0;
    {   // cfg->device is current here
        void* p = nullptr;
        const int rc = scratch_address(cfg->device, &p);
        if (rc != TOPK_ATTN_OK) { delete h; return rc; }
        h->scratch_dev = static_cast<char*>(p);
    }
    // lengths and the small per-head control words start at zero
    if (hipMemset(cfg->workspace, 0, w.hist) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        delete h;
        return TOPK_ATTN_EDEVICE;
    }
    *out = h;
    return TOPK_ATTN_OK;
}

int topk_attn_destroy(topk_attn_t* h) {
    if (!h) return TOPK_ATTN_EINVAL;
    for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
    delete h;
    return TOPK_ATTN_OK;
}

int64_t topk_attn_length(const topk_attn_t* h, int layer, int seq) {
    if (!h || layer < 0 || layer >= h->cfg.n_layers || seq < 0 || seq >= h->cfg.n_seqs) return -1;
    return h->len[(size_t)layer * h->cfg.n_seqs + seq];
}

int topk_attn_set_path(topk_attn_t* h, int path) {
    if (!h || path < TOPK_ATTN_PATH_AUTO || path > TOPK_ATTN_PATH_PAGES) return TOPK_ATTN_EINVAL;
    if (path == TOPK_ATTN_PATH_INDEX && h->cfg.index_kind != TOPK_ATTN_INDEX_INT8) return TOPK_ATTN_EINVAL;
    if (path == TOPK_ATTN_PATH_PAGES && h->cfg.index_kind != TOPK_ATTN_INDEX_PAGES) return TOPK_ATTN_EINVAL;
    h->path = path;
    return TOPK_ATTN_OK;
}

int topk_attn_reset(topk_attn_t* h, int layer, int seq, void* hip_stream) {
    if (!h || layer < 0 || layer >= h->cfg.n_layers || seq < 0 || seq >= h->cfg.n_seqs) return TOPK_ATTN_EINVAL;
    const size_t slot = (size_t)layer * h->cfg.n_seqs + seq;
    int32_t* len_dev = reinterpret_cast<int32_t*>(static_cast<char*>(h->cfg.workspace) + h->ws.len) + slot;
    hipLaunchKernelGGL(set_len_kernel, dim3(1), dim3(1), 0, (hipStream_t)hip_stream, len_dev, 0);
    if (hipGetLastError() != hipSuccess) return TOPK_ATTN_EDEVICE;
    h->len[slot] = 0;
    return TOPK_ATTN_OK;
}

int topk_attn_append_kv(topk_attn_t* h, int layer, int seq, const void* k_new, const void* v_new, int64_t n_new,
                        int64_t token_stride, int64_t head_stride, void* hip_stream) {
    if (!h || layer < 0 || layer >= h->cfg.n_layers || seq < 0 || seq >= h->cfg.n_seqs) return TOPK_ATTN_EINVAL;
    if (n_new < 0) return TOPK_ATTN_EINVAL;
    if (n_new == 0) return TOPK_ATTN_OK;
    if (!k_new || !v_new) return TOPK_ATTN_EINVAL;
    const topk_attn_config& c = h->cfg;
    const int e = elem_bytes(c.dtype);
    if (token_stride < 0 || head_stride < 0) return TOPK_ATTN_EINVAL;
    if (((uintptr_t)k_new | (uintptr_t)v_new) & 15) return TOPK_ATTN_EINVAL;
    if (((token_stride * e) | (head_stride * e)) & 15) return TOPK_ATTN_EINVAL;
    const size_t slot = (size_t)layer * c.n_seqs + seq;
    const int64_t cur = h->len[slot];
    if (cur + n_new > c.max_tokens) return TOPK_ATTN_ECAPACITY;

    const int64_t row_b = (int64_t)c.head_dim * e;
    const int64_t head_b = c.max_tokens * row_b;
    const int64_t off = ((int64_t)slot * c.n_kv_heads) * head_b + cur * row_b;
    char* kdst = static_cast<char*>(c.kv_storage) + off;
    char* vdst = static_cast<char*>(c.kv_storage) + h->kv_half + off;
    int32_t* len_dev = reinterpret_cast<int32_t*>(static_cast<char*>(c.workspace) + h->ws.len) + slot;
    const int chunks = (int)(row_b / 16);
    const int64_t total = n_new * c.n_kv_heads * chunks;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       static_cast<const char*>(k_new), static_cast<const char*>(v_new), kdst, vdst, n_new,
                       c.n_kv_heads, chunks, token_stride * e, head_stride * e, head_b, len_dev,
                       (int32_t)(cur + n_new));
    if (hipGetLastError() != hipSuccess) return TOPK_ATTN_EDEVICE;
    if (c.index_kind == TOPK_ATTN_INDEX_INT8) {   // code the rows just written (stream order: after the copy)
        char* base = static_cast<char*>(c.kv_storage) + 2 * h->kv_half;
        const int64_t row0 = (int64_t)slot * c.n_kv_heads * c.max_tokens + cur;
        int8_t* codes = reinterpret_cast<int8_t*>(base) + row0 * c.head_dim;
        float* scales = reinterpret_cast<float*>(base + index_codes_bytes(&c)) + row0;
        if (launch_quantize_rows(c.dtype, c.head_dim, kdst, n_new, head_b, c.n_kv_heads, codes, scales, c.max_tokens,
                                 (hipStream_t)hip_stream) != hipSuccess)
            return TOPK_ATTN_EDEVICE;
    }
    if (c.index_kind == TOPK_ATTN_INDEX_PAGES) {   // balls of the pages just touched (stream order: after the copy)
        char* base = static_cast<char*>(c.kv_storage) + 2 * h->kv_half;
        const int64_t pcap = page_cap_of(&c);
        const int64_t stream0 = (int64_t)slot * c.n_kv_heads;
        char* centres = base + stream0 * pcap * row_b;
        float* balls = reinterpret_cast<float*>(base + page_centres_bytes(&c)) + stream0 * pcap * 2;
        const char* kseq = static_cast<const char*>(c.kv_storage) + stream0 * head_b;
        if (launch_page_balls(c.dtype, c.head_dim, kseq, c.max_tokens, pcap, c.n_kv_heads, 1, nullptr, cur, n_new, centres,
                              balls, (hipStream_t)hip_stream) != hipSuccess)
            return TOPK_ATTN_EDEVICE;
    }
    h->len[slot] = cur + n_new;
    return TOPK_ATTN_OK;
}

int topk_attn_append_step(topk_attn_t* h, int layer, const void* k_new, const void* v_new, int64_t n_new,
                          void* hip_stream) {
    if (!h || layer < 0 || layer >= h->cfg.n_layers || n_new < 0) return TOPK_ATTN_EINVAL;
    if (n_new == 0) return TOPK_ATTN_OK;
    if (!k_new || !v_new || (((uintptr_t)k_new | (uintptr_t)v_new) & 15)) return TOPK_ATTN_EINVAL;
    const topk_attn_config& c = h->cfg;
    const int B = c.n_seqs;
    for (int b = 0; b < B; ++b)
        if (h->len[(size_t)layer * B + b] + n_new > c.max_tokens) return TOPK_ATTN_ECAPACITY;
    hipStream_t st = (hipStream_t)hip_stream;
    const int e = elem_bytes(c.dtype);
    const int64_t row_b = (int64_t)c.head_dim * e, head_b = c.max_tokens * row_b;
    const int64_t layer_off = (int64_t)layer * B * c.n_kv_heads * head_b;
    char* kdst = static_cast<char*>(c.kv_storage) + layer_off;
    char* vdst = static_cast<char*>(c.kv_storage) + h->kv_half + layer_off;
    int32_t* len_dev = reinterpret_cast<int32_t*>(static_cast<char*>(c.workspace) + h->ws.len) + (size_t)layer * B;
    const int chunks = (int)(row_b / 16);
    const int64_t total = (int64_t)B * n_new * c.n_kv_heads * chunks;
    if (c.index_kind == TOPK_ATTN_INDEX_NONE && total <= kAppendSmallPieces) {
        hipLaunchKernelGGL(append_step_small_kernel, dim3(1), dim3(kAppendSmallThreads), 0, st, static_cast<const char*>(k_new),
                           static_cast<const char*>(v_new), kdst, vdst, len_dev, total, n_new, c.n_kv_heads, chunks, head_b, B);
        if (hipGetLastError() != hipSuccess) return TOPK_ATTN_EDEVICE;
        for (int b = 0; b < B; ++b) h->len[(size_t)layer * B + b] += n_new;
        return TOPK_ATTN_OK;
    }
    if (c.index_kind == TOPK_ATTN_INDEX_INT8 && total <= kAppendSmallPieces) {      // the same with the rows' codes
        char* base = static_cast<char*>(c.kv_storage) + 2 * h->kv_half;
        const int64_t layer_rows = (int64_t)layer * B * c.n_kv_heads * c.max_tokens;
        int8_t* codes = reinterpret_cast<int8_t*>(base) + layer_rows * c.head_dim;
        float* scales = reinterpret_cast<float*>(base + index_codes_bytes(&c)) + layer_rows;
        if (launch_append_step_small8(c.dtype, c.head_dim, k_new, v_new, kdst, vdst, head_b, B, n_new, c.n_kv_heads,
                                      c.max_tokens, len_dev, codes, scales, st) != hipSuccess)
            return TOPK_ATTN_EDEVICE;
        for (int b = 0; b < B; ++b) h->len[(size_t)layer * B + b] += n_new;
        return TOPK_ATTN_OK;
    }
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(append_step_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const char*>(k_new),
                       static_cast<const char*>(v_new), kdst, vdst, len_dev, total, n_new, c.n_kv_heads, chunks, head_b);
    if (hipGetLastError() != hipSuccess) return TOPK_ATTN_EDEVICE;
    if (c.index_kind == TOPK_ATTN_INDEX_INT8) {
        char* base = static_cast<char*>(c.kv_storage) + 2 * h->kv_half;
        const int64_t layer_rows = (int64_t)layer * B * c.n_kv_heads * c.max_tokens;
        int8_t* codes = reinterpret_cast<int8_t*>(base) + layer_rows * c.head_dim;
        float* scales = reinterpret_cast<float*>(base + index_codes_bytes(&c)) + layer_rows;
        if (launch_quantize_step(c.dtype, c.head_dim, k_new, B, n_new, c.n_kv_heads, c.max_tokens, len_dev, codes, scales,
                                 st) != hipSuccess)
            return TOPK_ATTN_EDEVICE;
    }
    if (c.index_kind == TOPK_ATTN_INDEX_PAGES) {
        char* base = static_cast<char*>(c.kv_storage) + 2 * h->kv_half;
        const int64_t pcap = page_cap_of(&c);
        const int64_t stream0 = (int64_t)layer * B * c.n_kv_heads;
        char* centres = base + stream0 * pcap * row_b;
        float* balls = reinterpret_cast<float*>(base + page_centres_bytes(&c)) + stream0 * pcap * 2;
        if (launch_page_balls(c.dtype, c.head_dim, kdst, c.max_tokens, pcap, c.n_kv_heads, B, len_dev, 0, n_new, centres, balls,
                              st) != hipSuccess)
            return TOPK_ATTN_EDEVICE;
    }
    hipLaunchKernelGGL(bump_len_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, st, len_dev, B, (int32_t)n_new);
    if (hipGetLastError() != hipSuccess) return TOPK_ATTN_EDEVICE;
    for (int b = 0; b < B; ++b) h->len[(size_t)layer * B + b] += n_new;
    return TOPK_ATTN_OK;
}

static void fill_call(topk_attn_t* h, int layer, const void* q, int k, int n_queries, Shape* s, Bufs* b,
                      bool use_static = false) {
    const topk_attn_config& c = h->cfg;
    const int e = elem_bytes(c.dtype);
    s->Bc = c.n_seqs; s->M = n_queries; s->causal = 0; s->B = c.n_seqs * n_queries;
    s->Hq = c.n_q_heads; s->Hkv = c.n_kv_heads; s->G = c.n_q_heads / c.n_kv_heads;
    s->row_tiles = n_queries * s->G > 16 ? 2 : 1;
    s->n_qblk = (n_queries * s->G + 16 * s->row_tiles - 1) / (16 * s->row_tiles);
    s->D = c.head_dim; s->dtype = c.dtype; s->k = k; s->window = 0; s->max_k = c.max_k;
    s->hist_cap = h->ws.hist_cap; s->tail_spw = 1; s->tail_wgs = 1;
    s->cand_cap = h->ws.cand_cap; s->bnd_cap = h->ws.bnd_cap; s->n_seg = 4; s->seg_cap = (h->ws.cand_cap / 4) & ~(kCandChunk - 1); s->samp_cap = kSampMax; s->n_chunk_cap = h->ws.n_chunk_cap;
    s->Ncap = c.max_tokens;
    s->indexed = 0;
    s->paged = 0; s->no_rescan = 0;
    s->page_cap = (int)page_cap_of(&c); s->page_words = h->ws.page_words;
    s->force_redo = h->force_redo ? 1 : 0;
    char* const ws_len = static_cast<char*>(c.workspace);
    // everything after the lengths is per-call scratch: the handle's workspace, or the library's own array
    char* const ws = use_static ? reinterpret_cast<char*>(reinterpret_cast<uintptr_t>(h->scratch_dev) - h->ws.thr) : ws_len;
    const size_t layer_b = (size_t)c.n_seqs * c.n_kv_heads * (size_t)c.max_tokens * c.head_dim * e;
    b->K = static_cast<char*>(c.kv_storage) + (size_t)layer * layer_b;
    b->V = static_cast<char*>(c.kv_storage) + h->kv_half + (size_t)layer * layer_b;
    b->q = q;
    b->K8 = nullptr; b->Kscale = nullptr;
    if (c.index_kind == TOPK_ATTN_INDEX_INT8) {
        const char* base = static_cast<const char*>(c.kv_storage) + 2 * h->kv_half;
        const size_t layer_rows = (size_t)layer * c.n_seqs * c.n_kv_heads * (size_t)c.max_tokens;
        b->K8 = reinterpret_cast<const int8_t*>(base) + layer_rows * c.head_dim;
        b->Kscale = reinterpret_cast<const float*>(base + index_codes_bytes(&c)) + layer_rows;
    }
    b->page_centres = nullptr; b->page_balls = nullptr;
    if (c.index_kind == TOPK_ATTN_INDEX_PAGES) {
        const char* base = static_cast<const char*>(c.kv_storage) + 2 * h->kv_half;
        const size_t layer_streams = (size_t)layer * c.n_seqs * c.n_kv_heads;
        b->page_centres = base + layer_streams * (size_t)page_cap_of(&c) * c.head_dim * e;
        b->page_balls = reinterpret_cast<const float*>(base + page_centres_bytes(&c)) + layer_streams * (size_t)page_cap_of(&c) * 2;
    }
    b->page_mask = reinterpret_cast<uint64_t*>(ws + h->ws.page_mask);
    b->page_cnt = reinterpret_cast<uint32_t*>(ws + h->ws.page_cnt);
    b->page_list = reinterpret_cast<int32_t*>(ws + h->ws.page_list);
    b->q8 = reinterpret_cast<int8_t*>(ws + h->ws.q8);
    b->qscale = reinterpret_cast<float*>(ws + h->ws.qscale);
    b->len = reinterpret_cast<int32_t*>(ws_len + h->ws.len) + (size_t)layer * c.n_seqs;
    b->thr = reinterpret_cast<float*>(ws + h->ws.thr);
    b->bins = reinterpret_cast<float*>(ws + h->ws.bins);
    b->hist = reinterpret_cast<uint32_t*>(ws + h->ws.hist);
    b->bnd = reinterpret_cast<uint64_t*>(ws + h->ws.bnd);
    b->tailrec = reinterpret_cast<uint32_t*>(ws + h->ws.tailrec);
    b->samp = reinterpret_cast<float*>(ws + h->ws.samp);
    b->seg_cnt = reinterpret_cast<uint32_t*>(ws + h->ws.seg_cnt);
    b->seg_max = reinterpret_cast<float*>(ws + h->ws.seg_max);
    b->seg_cnt2 = reinterpret_cast<uint32_t*>(ws + h->ws.seg_cnt2);
    b->flags = reinterpret_cast<uint32_t*>(ws + h->ws.flags);
    b->hmax = reinterpret_cast<float*>(ws + h->ws.hmax);
    b->cand = reinterpret_cast<uint64_t*>(ws + h->ws.cand);
    b->scores = reinterpret_cast<float*>(ws + h->ws.scores);
    b->sel_idx = reinterpret_cast<int32_t*>(ws + h->ws.sel_idx);
    b->sel_val = reinterpret_cast<float*>(ws + h->ws.sel_val);
    b->part_acc = reinterpret_cast<float*>(ws + h->ws.part_acc);
    b->part_l = reinterpret_cast<float*>(ws + h->ws.part_l);
    b->part_m = reinterpret_cast<float*>(ws + h->ws.part_m);
    b->out = nullptr; b->lse = nullptr;
    b->fallback_total = reinterpret_cast<uint32_t*>(ws + h->ws.fallback);
}

// Split of each head's candidate list into per-wave segments for the filtered scan:
// about two 4-wave workgroups per compute unit over the whole grid, no more waves than
// key tiles, and segments large enough for their share of the expected candidates plus
// eight standard deviations.  False if no split fits (the caller takes the full path).
static bool choose_segments(const topk_attn_t* h, const Shape& s, int64_t nmax, int64_t c_hi, int* n_seg,
                            int* seg_cap) {
    const int64_t target_wgs = 2 * (int64_t)h->n_cu;
    int64_t P = target_wgs / ((int64_t)scan_grid_z(s) * s.Hkv);
    const int64_t tiles = (nmax + 63) / 64;
    if (P * 4 > tiles) P = tiles / 4;
    if (P * 4 > kMaxSeg) P = kMaxSeg / 4;
    if (P > s.hist_cap) P = s.hist_cap;     // every scan workgroup leaves its per-bin candidate counts
    if (P < 1) P = 1;
    while (P & (P - 1)) P &= P - 1;          // power of two: the selection indexes segments by mask
    {   // rounding down may leave the chip a quarter empty: take the next power of two if it stays within 1.5 x
        const int64_t streams = (int64_t)scan_grid_z(s) * s.Hkv;
        if (streams * P * 8 < target_wgs * 7 && streams * P * 2 * 2 <= target_wgs * 3 && P * 2 * 4 <= tiles &&
            P * 2 * 4 <= kMaxSeg && P * 2 <= s.hist_cap)
            P *= 2;
    }
    for (; P >= 1; P /= 2) {
        const int64_t ns = P * 4;
        const int64_t cap = (s.cand_cap / ns) & ~(int64_t)(kCandChunk - 1);
        const double mean = (double)c_hi / (double)ns;
        if ((double)cap >= mean + 8.0 * sqrt(mean) + 32.0) {
            *n_seg = (int)ns;
            *seg_cap = (int)cap;
            return true;
        }
        if (P == 1) break;
    }
    return false;
}

// Shortest and longest searched prefix over the sequences of a layer; EINVAL if a sequence is empty.
static int lengths_of(const topk_attn_t* h, int layer, int window, int64_t min_tokens, int64_t* nmin,
                      int64_t* nmax) {
    const int B = h->cfg.n_seqs;
    int64_t lo = INT64_MAX, hi = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = h->len[(size_t)layer * B + b];
        if (n < min_tokens) return TOPK_ATTN_EINVAL;
        const int64_t p = prefix_len(n, window);
        lo = p < lo ? p : lo;
        hi = p > hi ? p : hi;
    }
    *nmin = lo; *nmax = hi;
    return TOPK_ATTN_OK;
}

static int decode_impl(topk_attn_t* h, int layer, const void* q, int n_queries, int causal, int k, int window,
                       float* out, int32_t* idx, float* vals, float* lse, void* hip_stream, bool use_static = false) {
    if (!h || !q || !out) return TOPK_ATTN_EINVAL;
    if (use_static && h->ws.total - h->ws.thr > kStaticScratchBytes) return TOPK_ATTN_ESCRATCH;
    if (layer < 0 || layer >= h->cfg.n_layers) return TOPK_ATTN_EINVAL;
    if (k < 1 || k > h->cfg.max_k) return TOPK_ATTN_EINVAL;
    if (window < 0 || window > h->cfg.max_window) return TOPK_ATTN_EINVAL;
    if (n_queries < 1 || n_queries > (h->cfg.max_queries > 1 ? h->cfg.max_queries : 1)) return TOPK_ATTN_EINVAL;
    if (window > h->cfg.max_tokens) window = (int)h->cfg.max_tokens;   // same result: no sequence is longer
    if ((uintptr_t)q & 15) return TOPK_ATTN_EINVAL;
    // the plans below are made for the longest searched prefix of each sequence (its last
    // query's); the earlier queries of a causal chunk search up to n_queries - 1 keys fewer
    int64_t nmin, nmax;
    if (lengths_of(h, layer, window, causal ? n_queries : 1, &nmin, &nmax) != TOPK_ATTN_OK) return TOPK_ATTN_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    Shape s; Bufs b;
    fill_call(h, layer, q, k, n_queries, &s, &b, use_static);
    s.window = window;
    s.causal = causal ? 1 : 0;
    b.out = out; b.lse = lse;
    if (idx) b.sel_idx = idx;
    if (vals) b.sel_val = vals;

    // the int8 index serves one query per sequence with the grouped scan layout
    const bool want_index = h->path == TOPK_ATTN_PATH_INDEX && n_queries == 1 && s.G <= 4;
    s.indexed = want_index ? 1 : 0;
    // the page index serves the grouped scan (with a window: over the pages of the searched prefix)
    const bool want_pages = h->path == TOPK_ATTN_PATH_PAGES && n_queries == 1 && s.G <= 4;
    // The batch takes the filtered scan if its longest sequence is worth it.  Shorter sequences
    // ride along whenever their candidate list fits; the few that cannot be filtered at all (a
    // handful of tokens, or k too dense) are recognised by the kernels themselves (same
    // plan_is_fast) and go straight to the exact redo of the selection, which is cheap for them.
    bool fast = false;
    if (h->path != TOPK_ATTN_PATH_FULL && scan_mfma_supported(s) && nmax > 0) {
        const Plan longest = make_plan(nmax, k < nmax ? k : (int)nmax, s.indexed);
        int64_t total = 0;               // searched tokens of the whole call
        for (int i = 0; i < s.Bc; ++i) total += prefix_len(h->len[(size_t)layer * s.Bc + i], window);
        fast = plan_is_fast(longest, nmax, s.cand_cap, h->path == TOPK_ATTN_PATH_FILTER,
                            total >= kFilterBatchTokens ? kFilterMinNBatch : kFilterMinN);
        int64_t c_hi = 0;
        for (int i = 0; i < s.Bc && fast; ++i) {
            const int64_t n = prefix_len(h->len[(size_t)layer * s.Bc + i], window);
            if (n == 0) continue;            // this sequence lies entirely inside its window
            const Plan pl = make_plan(n, k < n ? k : (int)n, s.indexed);
            if (plan_is_fast(pl, n, s.cand_cap, true)) c_hi = pl.c_hi > c_hi ? pl.c_hi : c_hi;
        }
        if (fast) fast = choose_segments(h, s, nmax, c_hi, &s.n_seg, &s.seg_cap);
        if (fast) {     // tail: about 128 selected rows per workgroup and at most four scan workgroups each
            // (a tail workgroup walks its scan workgroups one after the other: dependent loads each time)
            const int n_wg = s.n_seg / 4;
            int want = (k + 127) / 128;
            if (want < (n_wg + 3) / 4) want = (n_wg + 3) / 4;
            want = want < 1 ? 1 : (want > n_wg ? n_wg : want);
            s.tail_spw = (n_wg + want - 1) / want;
            s.tail_wgs = (n_wg + s.tail_spw - 1) / s.tail_spw;
        }
    }
    if (!fast) s.indexed = 0;      // no filtered scan: exact path
    if (fast && s.indexed) s.no_rescan = 1;   // (the per-bin counts cover the listed candidates only: an unusable list is redone densely)
    // the selection that follows the filtered scan has limits of its own (count vectors, partial-sum slots); they hold
    // for every shape the scan takes with this workspace, and a shape beyond them takes the exact path like any other
    if (fast && !tail_supported(s)) { fast = false; s.indexed = 0; s.no_rescan = 0; }
    hipError_t e = hipSuccess;
    bool tail_done = false;
    if (use_static) {
        // the array keeps what the last call on this GPU left: the per-head control words start at zero
        // (a fill kernel, so that the call may be recorded into a HIP graph)
        uint32_t* first = b.flags;
        const size_t n_words = (size_t)(reinterpret_cast<char*>(b.fallback_total) + sizeof(uint32_t) -
                                        reinterpret_cast<char*>(first)) / sizeof(uint32_t);
        hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n_words + 255) / 256 < 64 ? (n_words + 255) / 256 : 64)),
                           dim3(256), 0, st, first, n_words);
        e = hipGetLastError();
    }
    const bool timed = h->timing && h->ev_used < kTimingSlots;
    if (fast && s.indexed) {
        e = launch_quantize_rows(s.dtype, s.D, q, (int64_t)s.B * s.Hq, 0, 1, b.q8, b.qscale, 0, st);
        if (e == hipSuccess) e = launch_scan8_sample(s, b, nmax, st);
        if (e == hipSuccess) e = launch_threshold(s, b, nmax, st);
        if (e == hipSuccess && timed) e = hipEventRecord(h->ev[2 * h->ev_used], st);
        if (e == hipSuccess) e = launch_scan8_filter(s, b, st);
        if (e == hipSuccess && timed) e = hipEventRecord(h->ev[2 * h->ev_used + 1], st);
        if (e == hipSuccess && timed) h->ev_used++;
        if (e == hipSuccess) e = launch_rerank(s, b, st);              // exact scores, and their per-bin counts for the tail
        if (e == hipSuccess) e = launch_tail(s, b, st);                // (with a window: its partial sums too)
        tail_done = true;
    } else if (fast) {
        s.paged = want_pages ? 1 : 0;
        s.no_rescan = s.paged;      // the paged scan deals its tiles to the waves by rank among the pages kept
        e = launch_scan_sample(s, b, nmax, st);
        if (e == hipSuccess) e = launch_threshold(s, b, nmax, st);
        if (e == hipSuccess && s.paged) e = launch_page_filter(s, b, h->page_beta, st);
        if (e == hipSuccess && timed) e = hipEventRecord(h->ev[2 * h->ev_used], st);
        if (e == hipSuccess) e = s.paged ? launch_scan_filter_paged(s, b, st) : launch_scan_filter(s, b, nmax, st);
        if (e == hipSuccess && timed) e = hipEventRecord(h->ev[2 * h->ev_used + 1], st);
        if (e == hipSuccess && timed) h->ev_used++;
        if (e == hipSuccess) e = launch_tail(s, b, st);                // selection and gather (with a window: its partial sums too); redoes unusable heads itself
        tail_done = true;
    } else {
        if (nmax > 0) {
            if (timed) e = hipEventRecord(h->ev[2 * h->ev_used], st);
            if (e == hipSuccess) e = launch_scan_full(s, b, nmax, b.scores, st);
            if (e == hipSuccess && timed) e = hipEventRecord(h->ev[2 * h->ev_used + 1], st);
            if (e == hipSuccess && timed) h->ev_used++;
        }
        if (e == hipSuccess) e = launch_select_full(s, b, nmax, st);   // with nothing to search it only pads
    }
    if (e == hipSuccess && !tail_done) e = launch_gather(s, b, st);
    h->last_fast = fast;
    h->last_paged = fast && s.paged;
    h->last_tail = tail_done;
    h->last_queries = n_queries;
    h->last_n_seg = fast ? s.n_seg : 0;
    h->last_seg_cap = fast ? s.seg_cap : 0;
    h->last_layer = layer;
    h->last_static = use_static;
    return e == hipSuccess ? TOPK_ATTN_OK : TOPK_ATTN_EDEVICE;
}

int topk_attn_decode(topk_attn_t* h, int layer, const void* q, int k, float* out, int32_t* idx, float* vals,
                     float* lse, void* hip_stream) {
    return decode_impl(h, layer, q, 1, 0, k, 0, out, idx, vals, lse, hip_stream);
}

int topk_attn_decode_static(topk_attn_t* h, int layer, const void* q, int k, float* out, int32_t* idx, float* vals,
                            float* lse, void* hip_stream) {
    return decode_impl(h, layer, q, 1, 0, k, 0, out, idx, vals, lse, hip_stream, true);
}

int topk_attn_decode_window(topk_attn_t* h, int layer, const void* q, int k, int window, float* out, int32_t* idx,
                            float* vals, float* lse, void* hip_stream) {
    return decode_impl(h, layer, q, 1, 0, k, window, out, idx, vals, lse, hip_stream);
}

int topk_attn_decode_multi(topk_attn_t* h, int layer, const void* q, int n_queries, int causal, int k, int window,
                           float* out, int32_t* idx, float* vals, float* lse, void* hip_stream) {
    return decode_impl(h, layer, q, n_queries, causal, k, window, out, idx, vals, lse, hip_stream);
}

int topk_attn_decode_layers(topk_attn_t* h, int layer0, int n_layers, const void* q, const int32_t* k, int window,
                            float* out, int32_t* idx, float* vals, float* lse, void* hip_stream) {
    if (!h || !q || !out || !k) return TOPK_ATTN_EINVAL;
    if (n_layers < 1 || layer0 < 0 || layer0 > h->cfg.n_layers - n_layers) return TOPK_ATTN_EINVAL;
    if (window < 0 || window > h->cfg.max_window || ((uintptr_t)q & 15)) return TOPK_ATTN_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if (k[l] < 1 || k[l] > h->cfg.max_k) return TOPK_ATTN_EINVAL;
        for (int b = 0; b < h->cfg.n_seqs; ++b)
            if (h->len[(size_t)(layer0 + l) * h->cfg.n_seqs + b] < 1) return TOPK_ATTN_EINVAL;
    }
    const size_t BH = (size_t)h->cfg.n_seqs * h->cfg.n_q_heads;
    const size_t q_step = BH * h->cfg.head_dim * elem_bytes(h->cfg.dtype);
    size_t sel_off = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int rc = decode_impl(h, layer0 + l, static_cast<const char*>(q) + l * q_step, 1, 0, k[l], window,
                                   out + l * BH * h->cfg.head_dim, idx ? idx + sel_off : nullptr,
                                   vals ? vals + sel_off : nullptr, lse ? lse + l * BH : nullptr, hip_stream);
        if (rc != TOPK_ATTN_OK) return rc;
        sel_off += BH * (size_t)k[l];
    }
    return TOPK_ATTN_OK;
}

int topk_attn_k_schedule(int64_t total_k, int n_layers, double last_over_first, int32_t* k_out) {
    if (!k_out || n_layers < 1 || total_k < n_layers) return TOPK_ATTN_EINVAL;
    if (!(last_over_first > 0.0) || !std::isfinite(last_over_first)) return TOPK_ATTN_EINVAL;
    std::vector<double> w((size_t)n_layers);
    double wsum = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        w[l] = n_layers == 1 ? 1.0 : 1.0 + (last_over_first - 1.0) * (double)l / (double)(n_layers - 1);
        wsum += w[l];
    }
    std::vector<int64_t> k((size_t)n_layers);
    std::vector<std::pair<double, int>> frac((size_t)n_layers);
    int64_t used = 0;
    for (int l = 0; l < n_layers; ++l) {
        const double exact = (double)total_k * w[l] / wsum;
        int64_t fl = (int64_t)floor(exact);
        if (fl < 1) fl = 1;                       // every layer attends to at least one key
        k[l] = fl;
        used += fl;
        frac[l] = {exact - (double)fl, l};
    }
    // hand out (or, after the >= 1 clamp, take back) the remainder by fractional part
    std::sort(frac.begin(), frac.end(), [](const std::pair<double, int>& a, const std::pair<double, int>& b) {
        return a.first != b.first ? a.first > b.first : a.second > b.second;
    });
    int64_t rem = total_k - used;
    for (int i = 0; rem > 0; i = (i + 1) % n_layers, --rem) k[frac[i].second] += 1;
    for (int i = n_layers - 1; rem < 0; i = (i + n_layers - 1) % n_layers) {
        if (k[frac[i].second] > 1) { k[frac[i].second] -= 1; ++rem; }
    }
    for (int l = 0; l < n_layers; ++l) {
        if (k[l] > INT32_MAX) return TOPK_ATTN_EINVAL;
        k_out[l] = (int32_t)k[l];
    }
    return TOPK_ATTN_OK;
}

int topk_attn_scores(topk_attn_t* h, int layer, const void* q, float* scores, void* hip_stream) {
    if (!h || !q || !scores) return TOPK_ATTN_EINVAL;
    if (layer < 0 || layer >= h->cfg.n_layers) return TOPK_ATTN_EINVAL;
    if ((uintptr_t)q & 15) return TOPK_ATTN_EINVAL;
    int64_t nmin, nmax;
    if (lengths_of(h, layer, 0, 1, &nmin, &nmax) != TOPK_ATTN_OK) return TOPK_ATTN_EINVAL;
    Shape s; Bufs b;
    fill_call(h, layer, q, 1, 1, &s, &b);
    hipError_t e;
    if (h->path == TOPK_ATTN_PATH_INDEX && s.G <= 4) {   // approximate scores from the codes
        e = launch_quantize_rows(s.dtype, s.D, q, (int64_t)s.B * s.Hq, 0, 1, b.q8, b.qscale, 0, (hipStream_t)hip_stream);
        if (e == hipSuccess) e = launch_scan8_full(s, b, nmax, scores, (hipStream_t)hip_stream);
    } else {
        e = launch_scan_full(s, b, nmax, scores, (hipStream_t)hip_stream);
    }
    return e == hipSuccess ? TOPK_ATTN_OK : TOPK_ATTN_EDEVICE;
}

int topk_attn_last_fallbacks(topk_attn_t* h, int* n_heads) {
    if (!h || !n_heads) return TOPK_ATTN_EINVAL;
    *n_heads = 0;
    if (!h->last_fast) return TOPK_ATTN_OK;
    uint32_t v = 0;
    const char* where = h->last_static ? h->scratch_dev + (h->ws.fallback - h->ws.thr)
                                       : static_cast<char*>(h->cfg.workspace) + h->ws.fallback;
    if (hipMemcpy(&v, where, sizeof v, hipMemcpyDeviceToHost) !=
        hipSuccess)
        return TOPK_ATTN_EDEVICE;
    *n_heads = (int)v;
    return TOPK_ATTN_OK;
}

int topk_attn_set_page_bound_scale(topk_attn_t* h, float beta) {
    if (!h || h->cfg.index_kind != TOPK_ATTN_INDEX_PAGES || !(beta > 0.0f) || beta > 1.0f) return TOPK_ATTN_EINVAL;
    h->page_beta = beta;
    return TOPK_ATTN_OK;
}

int topk_attn_last_pages_read(topk_attn_t* h, int64_t* pages_read, int64_t* pages_total) {
    if (!h || !pages_read || !pages_total) return TOPK_ATTN_EINVAL;
    const topk_attn_config& c = h->cfg;
    int64_t total = 0;
    for (int b = 0; b < c.n_seqs; ++b) total += (h->len[(size_t)h->last_layer * c.n_seqs + b] + 63) / 64 * c.n_kv_heads;
    *pages_total = total;
    *pages_read = total;                       // every page, unless the last decode went through the page index
    if (!h->last_paged || h->last_static) return TOPK_ATTN_OK;
    const size_t words = (size_t)c.n_seqs * c.n_kv_heads * h->ws.page_words;
    std::vector<uint64_t> mask(words);
    if (hipMemcpy(mask.data(), static_cast<char*>(c.workspace) + h->ws.page_mask, words * sizeof(uint64_t),
                  hipMemcpyDeviceToHost) != hipSuccess)
        return TOPK_ATTN_EDEVICE;
    int64_t read = 0;
    for (uint64_t w : mask) read += __builtin_popcountll(w);
    *pages_read = read;
    return TOPK_ATTN_OK;
}

int topk_attn_last_selection_records(topk_attn_t* h, uint32_t* records) {
    if (!h || !records || !h->last_tail || h->last_static) return TOPK_ATTN_EINVAL;
    const topk_attn_config& c = h->cfg;
    const size_t n = (size_t)c.n_seqs * h->last_queries * c.n_q_heads;
    if (hipMemcpy(records, static_cast<char*>(c.workspace) + h->ws.tailrec, n * 4 * sizeof(uint32_t), hipMemcpyDeviceToHost) !=
        hipSuccess)
        return TOPK_ATTN_EDEVICE;
    std::vector<uint32_t> flags(n);
    if (hipMemcpy(flags.data(), static_cast<char*>(c.workspace) + h->ws.flags, n * sizeof(uint32_t), hipMemcpyDeviceToHost) !=
        hipSuccess)
        return TOPK_ATTN_EDEVICE;
    for (size_t i = 0; i < n; ++i) records[4 * i] |= flags[i] << 8;      // the head's flag word above the state
    return TOPK_ATTN_OK;
}

int topk_attn_debug_read_workspace(topk_attn_t* h, const char* name, void* dst, size_t bytes) {
    if (!h || !name || !dst) return TOPK_ATTN_EINVAL;
    const WsLayout& w = h->ws;
    const struct { const char* name; size_t at, end; } arrays[] = {
        {"thr", w.thr, w.bins}, {"bins", w.bins, w.samp}, {"samp", w.samp, w.seg_cnt}, {"seg_cnt", w.seg_cnt, w.seg_max},
        {"seg_max", w.seg_max, w.seg_cnt2}, {"seg_cnt2", w.seg_cnt2, w.flags}, {"flags", w.flags, w.hmax},
        {"tailrec", w.tailrec, w.qscale}, {"page_mask", w.page_mask, w.page_cnt}, {"page_cnt", w.page_cnt, w.page_list},
        {"page_list", w.page_list, w.hist}, {"hist", w.hist, w.cand}, {"cand", w.cand, w.bnd}, {"bnd", w.bnd, w.scores}};
    for (const auto& a : arrays) {
        if (strcmp(a.name, name) != 0) continue;
        if (bytes > a.end - a.at) return TOPK_ATTN_EINVAL;
        return hipMemcpy(dst, static_cast<char*>(h->cfg.workspace) + a.at, bytes, hipMemcpyDeviceToHost) == hipSuccess
                   ? TOPK_ATTN_OK : TOPK_ATTN_EDEVICE;
    }
    return TOPK_ATTN_EINVAL;
}

int topk_attn_debug_read_workspace_dims(topk_attn_t* h, int32_t* dims) {
    if (!h || !dims) return TOPK_ATTN_EINVAL;
    dims[0] = h->ws.cand_cap; dims[1] = h->ws.bnd_cap; dims[2] = h->ws.hist_cap; dims[3] = kMaxSeg;
    dims[4] = h->last_n_seg; dims[5] = h->last_seg_cap;
    return TOPK_ATTN_OK;
}

int topk_attn_debug_force_redo(topk_attn_t* h, int enable) {
    if (!h) return TOPK_ATTN_EINVAL;
    h->force_redo = enable != 0;
    return TOPK_ATTN_OK;
}

int topk_attn_set_scan_timing(topk_attn_t* h, int enable) {
    if (!h) return TOPK_ATTN_EINVAL;
    if (enable && h->ev.empty()) {
        h->ev.resize(2 * kTimingSlots);
        for (size_t i = 0; i < h->ev.size(); ++i) {
            if (hipEventCreate(&h->ev[i]) != hipSuccess) {
                for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(h->ev[j]);
                h->ev.clear();
                return TOPK_ATTN_EDEVICE;
            }
        }
    }
    h->timing = enable != 0;
    h->ev_used = 0;
    return TOPK_ATTN_OK;
}

int topk_attn_scan_time(topk_attn_t* h, double* total_ms, int* n_calls) {
    if (!h || !total_ms || !n_calls) return TOPK_ATTN_EINVAL;
    double sum = 0.0;
    for (int i = 0; i < h->ev_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, h->ev[2 * i], h->ev[2 * i + 1]) != hipSuccess) return TOPK_ATTN_EDEVICE;
        sum += ms;
    }
    *total_ms = sum;
    *n_calls = h->ev_used;
    h->ev_used = 0;
    return TOPK_ATTN_OK;
}

int topk_attn_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream) {
    if (!src || !sink || bytes == 0 || (bytes & 15) || ((uintptr_t)src & 15)) return TOPK_ATTN_EINVAL;
    const size_t n_vec = bytes / 16;
    size_t blocks = (n_vec + 4095) / 4096;      // one tile per wave at least
    if (blocks > 512) blocks = 512;             // two workgroups per compute unit, like the key scan
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       static_cast<const u32x4*>(src), n_vec, static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? TOPK_ATTN_OK : TOPK_ATTN_EDEVICE;
}

#ifndef TKA_BUILD_ID
#define TKA_BUILD_ID "unknown"
#endif
// the tag in front lets a script find the identifier in the file without loading it
static const char kBuildTag[] = "tka-build-id:" TKA_BUILD_ID;
const char* topk_attn_build_id(void) { return kBuildTag + 13; }

const char* topk_attn_strerror(int code) {
    switch (code) {
        case TOPK_ATTN_OK: return "ok";
        case TOPK_ATTN_EINVAL: return "invalid argument";
        case TOPK_ATTN_ECAPACITY: return "cache capacity exceeded";
        case TOPK_ATTN_EUNSUPPORTED: return "unsupported configuration";
        case TOPK_ATTN_EDEVICE: return "HIP error";
        case TOPK_ATTN_ENOMEM: return "out of memory or buffer too small";
        case TOPK_ATTN_ESCRATCH: return "configuration needs more per-call scratch than the library's built-in buffer holds";
        default: return "unknown error";
    }
}

}  // extern "C"
