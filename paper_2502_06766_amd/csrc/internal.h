// Internal declarations shared by the translation units of libtopk_attn (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tka {

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

constexpr int kWave = 64;
constexpr int kSelThreads = 1024;   // workgroup size of the selection kernels
constexpr int kGatherRows = 256;    // value rows handled by one gather workgroup
// Most sample scores per head in the threshold estimate.  The sample rows are random 256-byte reads
// (4.8 TB/s at best): 16384 per KV head cost 13 us at one million tokens, 8192 cost 9, for a sixth more
// candidates (the rank rule keeps the threshold six standard deviations below the expected k-th score).
constexpr int kSampMax = 8192;
constexpr int kSampMin = 1024;
// Shortest cache the filtered scan is used for unless forced: below, writing all scores and
// selecting over them is faster (measured crossovers: one sequence 16k tokens 46 against 56 us,
// 30k tokens 72 against 65 us; in a batch the small kernels of the filtered path are shared by
// more work and it wins from 8k tokens on once the call holds 128k tokens in all).
constexpr int kFilterMinN = 24576;
constexpr int kFilterMinNBatch = 8192;
constexpr int64_t kFilterBatchTokens = 131072;
constexpr int kMaxSeg = 1024;       // most candidate segments per head

// Geometry of one decode call, passed by value to every kernel.
struct Shape {
    int B;            // sequences of the call: B = Bc * M, sequence b is query b % M of cache sequence b / M
    int Hq, Hkv, G, D, dtype;
    int Bc;           // cache sequences
    int M;            // queries per cache sequence in this call (1 for plain decode)
    int causal;       // query m of M sees only the first len - (M - 1 - m) tokens
    int row_tiles;    // row-tile scan: 16-row tiles per pass over the keys (1 or 2)
    int n_qblk;       // row-tile scan: blocks of 16 * row_tiles (query, head) rows per KV head
    int indexed;      // the scan reads the int8 key index; candidates are re-scored exactly afterwards
    int force_redo;   // measurement aid: treat every head as not filterable (exact redo of all heads)
    int paged;        // the scan skips the pages the coarse page index rules out
    int no_rescan;    // an unusable list is redone densely (the per-bin counts of a paged scan are not those of the plain tile order)
    int page_cap;     // pages per key stream the page index has room for (ceil(Ncap / 64))
    int page_words;   // 64-bit words of the page mask per key stream
    int k;            // requested k (k_eff = min(k, searched prefix of sequence b))
    int window;       // most recent tokens that are always attended and excluded from the search
    int max_k;
    int cand_cap;     // entries per (b, head) candidate list
    int bnd_cap;      // entries per (b, head) boundary list
    int n_seg;        // segments the candidate list is split in (one per scanning wave), power of 2
    int seg_cap;      // entries per segment (n_seg * seg_cap <= cand_cap), a multiple of kCandChunk
    int samp_cap;     // entries per (b, head) sample-score row
    int n_chunk_cap;  // partial-sum slots per (b, head)
    int hist_cap;     // scan workgroups per head the per-bin candidate counts have room for
    int tail_spw;     // tail: scan workgroups whose candidates one tail workgroup takes
    int tail_wgs;     // tail: workgroups per head = ceil((n_seg / 4) / tail_spw)
    int64_t Ncap;     // row capacity per (layer, seq, kv head)
};

// Device pointers of one decode call.
struct Bufs {
    const void* K;          // this layer's keys  [B][Hkv][Ncap][D]
    const void* V;          // this layer's values
    const void* q;          // [B][Hq][D]
    const int8_t* K8;       // this layer's int8 key codes [Bc][Hkv][Ncap][D] (compressed index), or null
    const float* Kscale;    // this layer's per-row code scales [Bc][Hkv][Ncap]
    int8_t* q8;             // [B*Hq][D] query codes of this call
    float* qscale;          // [B*Hq]
    const int32_t* len;     // [Bc] tokens cached per cache sequence (this layer)
    float* thr;             // [B*Hq] candidate threshold
    float* bins;            // [B*Hq][2] lower end and bins per unit of score of tail_bin()
    float* samp;            // [B*Hq][samp_cap]
    uint32_t* seg_cnt;      // [B*Hq][n_seg] candidates each scanning wave found (may exceed seg_cap)
    float* seg_max;         // [B*Hq][n_seg] largest score each scanning wave saw (-inf if it saw none)
    uint32_t* seg_cnt2;     // [B*Hq][n_seg] lengths of the segments the tail fills again for a head whose list was unusable
    uint32_t* flags;        // [B*Hq] bit 0: the filter is not expected to work for the head's sequence (not a fallback if it does not);
                            // bit 1: set by the tail when keys sorted again did not fit their segments; bit 2: ignore a usable list
    float* hmax;            // [B*Hq] largest selected score
    uint64_t* cand;         // [B*Hq][cand_cap] (score bits << 32 | position); entry e of segment g
                            // at [cand_slot(e, g, n_seg)]
    uint32_t* hist;         // [B*Hq][hist_cap][kTailBins] candidates per score bin found by each scan workgroup
    uint64_t* bnd;          // [B*Hq][bnd_cap] candidates of the bin the k-th score falls in
    uint32_t* tailrec;      // [B*Hq][4] what the tail's second kernel needs to know of a head (TailRec)
    const void* page_centres;  // this layer's page centres [Bc][Hkv][page_cap][D] (cache dtype), or null
    const float* page_balls;   // this layer's [Bc][Hkv][page_cap][2]: radius of the page's ball, norm of its centre
    uint64_t* page_mask;       // [B][Hkv][page_words] one bit per page: 1 = the scan reads it
    uint32_t* page_cnt;        // [B][Hkv] pages the scan reads
    int32_t* page_list;        // [B][Hkv][64 * page_words] their numbers, ascending
    float* scores;          // [B*Hq][Ncap] full score buffer
    int32_t* sel_idx;       // [B*Hq][k]
    float* sel_val;         // [B*Hq][k]
    float* part_acc;        // [B*Hq][n_chunk_cap][D]
    float* part_l;          // [B*Hq][n_chunk_cap]
    float* part_m;          // [B*Hq][n_chunk_cap] score the partial's weights are relative to
    float* out;             // [B*Hq][D]
    float* lse;             // [B*Hq] or null
    uint32_t* fallback_total; // [1]
};

// The MFMA scan has two kernels: one query and at most four heads per KV head go through
// the grouped kernel (grid z = sequences), everything else through the row-tile kernel
// (grid z = cache sequences x row blocks).
inline bool scan_row_tiles(const Shape& s) { return s.M > 1 || s.G > 4; }
inline int scan_grid_z(const Shape& s) { return scan_row_tiles(s) ? s.Bc * s.n_qblk : s.B; }

// Cache sequence behind sequence b of the call, and the tokens of it that b may attend to.
__device__ inline int cache_seq(const Shape& sh, int b) { return sh.M == 1 ? b : b / sh.M; }
__device__ inline int64_t visible_len(const Shape& sh, const Bufs& bf, int b) {
    if (sh.M == 1) return bf.len[b];
    const int c = b / sh.M;
    return (int64_t)bf.len[c] - (sh.causal ? sh.M - 1 - (b - c * sh.M) : 0);
}

// Candidate list of one head: n_seg segments (one per scanning wave).  Runs of kCandChunk
// consecutive entries of a segment are contiguous (a wave's flush writes whole 128-byte
// pieces), and the runs of the segments interleave, so that the filled part of the list is
// dense at its start whatever the fill of the single segments.
constexpr int kCandChunkLog2 = 4;
constexpr int kCandChunk = 1 << kCandChunkLog2;
// slot of entry e of segment g
__host__ __device__ inline int64_t cand_slot(int64_t e, int g, int n_seg) {
    return ((((e >> kCandChunkLog2) * n_seg) + g) << kCandChunkLog2) | (e & (kCandChunk - 1));
}
// segment and entry of slot i (n_seg = 1 << log2_n_seg)
__host__ __device__ inline int cand_slot_segment(int64_t i, int log2_n_seg) {
    return (int)((i >> kCandChunkLog2) & ((1 << log2_n_seg) - 1));
}
__host__ __device__ inline int64_t cand_slot_entry(int64_t i, int log2_n_seg) {
    return (((i >> kCandChunkLog2) >> log2_n_seg) << kCandChunkLog2) | (i & (kCandChunk - 1));
}

// Coarse order of the candidates of a head by score, for the tail of the filtered path:
// bin 0 takes everything below `lo`, bins 1 .. kTailBins - 2 are 1 / inv_d wide from `lo`
// up, the last one is open-ended.  The threshold kernel lays the fine bins over the band of
// scores in which the sample puts the k-th largest score, so that the bin it falls in holds
// few candidates.  Monotone in the score; the scan (which counts candidates per bin) and the
// tail (which sorts them by bin) evaluate exactly this sequence of roundings.
constexpr int kTailBins = 64;
__device__ __forceinline__ int tail_bin(float score, float lo, float inv_d) {
    const float t = __fmul_rn(__fsub_rn(score, lo), inv_d);
    const int b = 1 + (int)fminf(t, (float)(kTailBins - 2));     // NaN (inf * 0) counts as the last bin
    return score < lo ? 0 : b;
}

// Tokens of a sequence the search runs over: everything but the always-attended window.
__host__ __device__ inline int64_t prefix_len(int64_t n_tokens, int window) {
    return n_tokens - (window < n_tokens ? (int64_t)window : n_tokens);
}

// Sampling plan for the threshold estimate of one sequence (same code on host and device).
struct Plan {
    int n_samp;      // sample keys per KV head (multiple of 64)
    int stride;      // one sample per `stride` consecutive positions
    int rank;        // threshold = rank-th largest sample score
    int rank_k;      // sample scores expected at or above the true k-th score (rounded up)
    int rank_lo;     // the k-th score lies between the sample scores of these two ranks
    int rank_hi;     // (rank_hi <= rank_k <= rank_lo <= rank) unless a four-sigma sampling event happens
    int64_t c_hi;    // candidates expected at most (z-sigma above the mean)
};

// `indexed`: the sample scores are approximate (int8 index); a quarter more samples are
// expected above the threshold so that coding noise at the k-th score stays inside the list.
__host__ __device__ inline Plan make_plan(int64_t N, int k_eff, int indexed = 0) {
    Plan p;
    int64_t ns = N / 64;
    if (ns > kSampMax) ns = kSampMax;
    if (ns < kSampMin) ns = kSampMin;
    if (ns > N) ns = N;
    ns &= ~int64_t(63);
    if (ns < 64) ns = 64;
    p.n_samp = (int)ns;
    p.stride = (int)(N / ns);
    if (p.stride < 1) p.stride = 1;
    // With r0 samples expected above the true k-th score, take the rank r solving
    // r - z sqrt(r) = r0 so that the threshold is below the k-th score unless a
    // z-sigma event happens; the candidate list then holds about N r / n_samp entries.
    const double z = 6.0;
    const double r_true = (double)k_eff * (double)ns / (double)N;
    double r0 = r_true;
    if (indexed) r0 = 1.25 * r0 + 4.0;      // approximate scores: more candidates, so that coding noise loses none
    double sr = 0.5 * (z + sqrt(z * z + 4.0 * r0));
    double r = sr * sr;
    p.rank = (int)r + 2;
    p.rank_k = (int)r0 + 1;
    p.rank_lo = (int)(r0 + 4.0 * sqrt(r0)) + 2;
    if (p.rank_lo > p.rank) p.rank_lo = p.rank;
    p.rank_hi = (int)(r_true - 4.0 * sqrt(r_true));     // (the band of the k-th score itself, also with an index)
    if (p.rank_hi < 1) p.rank_hi = 1;
    p.c_hi = (int64_t)((double)N * (r + z * sr + 2.0) / (double)ns) + 64;
    return p;
}

// The filtered scan needs the candidate list to fit; unless forced it is also skipped
// for short caches and for selections so dense that nearly every key would be a candidate
// (measured at 512k tokens: it wins up to k = 60 % of the cache, loses from 75 % on).
__host__ __device__ inline bool plan_is_fast(const Plan& p, int64_t N, int cand_cap, bool force,
                                             int64_t min_n = kFilterMinN) {
    if (N < 256 || p.rank > p.n_samp || p.c_hi > cand_cap) return false;
    return force || (N >= min_n && p.c_hi * 5 <= N * 4);
}

// Position of sample s: one jittered position inside each stride-long stratum.
__host__ __device__ inline int64_t sample_pos(int s, int stride) {
    uint32_t h = (uint32_t)s * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    return (int64_t)s * stride + (int64_t)(h % (uint32_t)stride);
}

// Launch wrappers (each returns the hipError_t of the launch).
hipError_t launch_scan_sample(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st);
hipError_t launch_scan_filter(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st);
hipError_t launch_scan_full(const Shape& s, const Bufs& b, int64_t Nmax, float* dst, hipStream_t st);
bool scan_mfma_supported(const Shape& s);

hipError_t launch_threshold(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st);
hipError_t launch_select_full(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st);

hipError_t launch_gather(const Shape& s, const Bufs& b, hipStream_t st);

// fused selection + gather after a filtered scan that counted its candidates per score bin
bool tail_supported(const Shape& s);
hipError_t launch_tail(const Shape& s, const Bufs& b, hipStream_t st);

// coarse page index
bool pages_supported(int dtype, int D, int G);
hipError_t launch_page_balls(int dtype, int D, const void* K, int64_t Ncap, int64_t Pcap, int Hkv, int B,
                             const int32_t* len_dev, int64_t row0, int64_t n_new, void* centres, float* balls, hipStream_t st);
hipError_t launch_page_filter(const Shape& s, const Bufs& b, float beta, hipStream_t st);
hipError_t launch_scan_filter_paged(const Shape& s, const Bufs& b, hipStream_t st);

// int8 key index
bool index8_supported(int dtype, int D, int G);
hipError_t launch_quantize_rows(int dtype, int D, const void* src, int64_t rows_per_head, int64_t src_head_stride_bytes,
                                int n_heads, int8_t* dst, float* scale, int64_t dst_head_stride_rows, hipStream_t st);
hipError_t launch_append_step_small8(int dtype, int D, const void* ksrc, const void* vsrc, void* kdst, void* vdst,
                                     int64_t head_bytes, int B, int64_t n_new, int Hkv, int64_t Ncap, int32_t* len,
                                     int8_t* codes, float* scale, hipStream_t st);
hipError_t launch_quantize_step(int dtype, int D, const void* src, int B, int64_t n_new, int Hkv, int64_t Ncap,
                                const int32_t* len, int8_t* codes, float* scale, hipStream_t st);
hipError_t launch_scan8_sample(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st);
hipError_t launch_scan8_filter(const Shape& s, const Bufs& b, hipStream_t st);
hipError_t launch_scan8_full(const Shape& s, const Bufs& b, int64_t Nmax, float* dst, hipStream_t st);
hipError_t launch_rerank(const Shape& s, const Bufs& b, hipStream_t st);

}  // namespace tka
