// Exact top-k selection (the result of the paper's knn_search: the k largest scores
// `vals` and their positions `I`), by radix select on unique 64-bit keys
// (order-preserving image of the fp32 score, then inverted position), so that equal
// scores resolve to the lower position and the selected set never depends on the order
// in which candidates were produced.  One workgroup per (sequence, head).
//
// The first CPT * kSelThreads items of a head are held in registers for all passes; anything
// beyond is re-read from memory in batches of independent loads.  Output order is fixed
// (thread-major), so repeated calls return bit-identical results.
#include "device_utils.h"
#include "internal.h"

namespace tka {

constexpr int kSelWaves = kSelThreads / kWave;
#ifndef TKA_DIGIT_BITS
#define TKA_DIGIT_BITS 9
#endif
constexpr int kDigitBits = TKA_DIGIT_BITS;     // radix digit width
constexpr int kBins = 1 << kDigitBits;
constexpr int kBinsPerLane = kBins / kWave;

struct SelShared {
    uint32_t hist[kBins];
    uint64_t red_max[kSelWaves];
    uint64_t red_min[kSelWaves];
    uint64_t bc_max, bc_min;
    uint32_t bin, above, cb;
    uint32_t wave_tot[kSelWaves];
    uint32_t scan_total;
    uint32_t seg_len[kMaxSeg];
};

// Sources of (score, position) items, split into "is there an item in slot i", "where is
// it" and "turn the loaded word into a key", so that a batch of independent loads can be
// issued before any of them is consumed.  Key 0 never occurs for a real item (its low
// word would have to be 0xFFFFFFFF - position = 0) and marks an empty slot.
struct SrcDense {            // scores[i], position i, i < n
    const float* s;
    int64_t n;
    typedef float raw_t;
    __device__ __forceinline__ int64_t slots() const { return n; }
    __device__ __forceinline__ bool valid(int64_t i) const { return i < n; }
    __device__ __forceinline__ const float* where(int64_t i) const { return s + i; }
    __device__ __forceinline__ uint64_t key(float r, int64_t i) const { return composite(r, (uint32_t)i); }
};
struct SrcSeg {              // candidate list of n_seg interleaved segments: entry e of segment g
    const uint64_t* segs;    // sits in slot e * n_seg + g; entries are (score bits << 32 | position)
    const uint32_t* seg_len; // LDS: entries per segment
    int n_seg;               // power of two
    int max_len;             // longest segment
    typedef uint64_t raw_t;
    __device__ __forceinline__ int64_t slots() const { return (int64_t)n_seg * max_len; }
    __device__ __forceinline__ bool valid(int64_t i) const {
        return i < slots() && (uint32_t)(i / n_seg) < seg_len[i & (n_seg - 1)];
    }
    __device__ __forceinline__ const uint64_t* where(int64_t i) const { return segs + i; }
    __device__ __forceinline__ uint64_t key(uint64_t e, int64_t) const {
        return composite(__uint_as_float((uint32_t)(e >> 32)), (uint32_t)e);
    }
};

// The items of one head as seen by one thread: register slot j holds slot
// j * kSelThreads + tid of the source, later slots are streamed.  Every lane of a wave visits the
// same slots in the same order (with a per-lane "present" flag), so callers may use
// wave-wide ballots inside the visitor.
template <int CPT, class Src>
struct Items {
    uint64_t kc[CPT > 0 ? CPT : 1];
    const Src& src;
    __device__ __forceinline__ Items(const Src& s) : src(s) {
        constexpr int B = CPT < 8 ? (CPT > 0 ? CPT : 1) : 8;     // independent loads per batch
#pragma unroll
        for (int j0 = 0; j0 < CPT; j0 += B) {
            typename Src::raw_t r[B];
            bool ok[B];
#pragma unroll
            for (int u = 0; u < B; ++u) {
                if (j0 + u < CPT) {          // CPT need not be a multiple of the batch
                    const int64_t i = (int64_t)(j0 + u) * kSelThreads + threadIdx.x;
                    ok[u] = src.valid(i);
                    r[u] = *src.where(ok[u] ? i : 0);
                }
            }
#pragma unroll
            for (int u = 0; u < B; ++u) {
                if (j0 + u < CPT) {
                    const int64_t i = (int64_t)(j0 + u) * kSelThreads + threadIdx.x;
                    kc[j0 + u] = ok[u] ? src.key(r[u], i) : 0ull;
                }
            }
        }
    }
    // f(key, present) for every slot, all lanes in lock step
    template <class F>
    __device__ __forceinline__ void for_each_sync(F f) const {
#pragma unroll
        for (int j = 0; j < CPT; ++j) f(kc[j], kc[j] != 0ull);
        constexpr int U = 8;
        const int64_t n_slots = src.slots();
        for (int64_t base = (int64_t)CPT * kSelThreads; base < n_slots; base += (int64_t)U * kSelThreads) {
            typename Src::raw_t r[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = base + (int64_t)u * kSelThreads + threadIdx.x;
                ok[u] = src.valid(i);
                r[u] = *src.where(ok[u] ? i : 0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = base + (int64_t)u * kSelThreads + threadIdx.x;
                f(ok[u] ? src.key(r[u], i) : 0ull, ok[u]);
            }
        }
    }
    template <class F>
    __device__ __forceinline__ void for_each(F f) const {
        for_each_sync([&](uint64_t c, bool present) { if (present) f(c); });
    }
};

// exclusive prefix sum of one value per thread over the workgroup; *total gets the sum
__device__ __forceinline__ uint32_t wg_exclusive_scan(uint32_t v, SelShared& sm, uint32_t* total) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t incl = v;
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += t;
    }
    __syncthreads();                      // protects wave_tot against a previous use
    if (lane == kWave - 1) sm.wave_tot[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        uint32_t w = lane < kSelWaves ? sm.wave_tot[lane] : 0u;
        uint32_t wi = w;
        for (int o = 1; o < kSelWaves; o <<= 1) {
            const uint32_t t = __shfl_up(wi, o, kWave);
            if (lane >= o) wi += t;
        }
        if (lane < kSelWaves) sm.wave_tot[lane] = wi - w;
        if (lane == kSelWaves - 1) sm.scan_total = wi;
    }
    __syncthreads();
    *total = sm.scan_total;
    return sm.wave_tot[wave] + incl - v;
}

// Returns T such that exactly k of the n items have key >= T (1 <= k <= n).
// *kmax receives the largest key.  All threads of the workgroup must call it.
template <class It>
__device__ uint64_t wg_select_kth(const It& items, int64_t n, int64_t k, SelShared& sm, uint64_t* kmax) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    uint64_t mx = 0, mn = ~0ull;
    items.for_each([&](uint64_t c) {
        mx = c > mx ? c : mx;
        mn = c < mn ? c : mn;
    });
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t a = __shfl_xor(mx, o, kWave), b = __shfl_xor(mn, o, kWave);
        mx = a > mx ? a : mx;
        mn = b < mn ? b : mn;
    }
    if (lane == 0) { sm.red_max[wave] = mx; sm.red_min[wave] = mn; }
    for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
    __syncthreads();
    if (wave == 0) {
        mx = lane < kSelWaves ? sm.red_max[lane] : 0ull;
        mn = lane < kSelWaves ? sm.red_min[lane] : ~0ull;
        for (int o = 32; o > 0; o >>= 1) {
            const uint64_t a = __shfl_xor(mx, o, kWave), b = __shfl_xor(mn, o, kWave);
            mx = a > mx ? a : mx;
            mn = b < mn ? b : mn;
        }
        if (lane == 0) { sm.bc_max = mx; sm.bc_min = mn; }
    }
    __syncthreads();
    mx = sm.bc_max; mn = sm.bc_min;
    *kmax = mx;
    if (k >= n) return mn;
    if (k == 1) return mx;

    // bits above `rb` are common to every remaining item and fixed in `prefix`
    int rb = 64 - __clzll((long long)(mx ^ mn));   // mx != mn: keys are unique and n >= 3 here
    uint64_t prefix = rb >= 64 ? 0ull : (mx >> rb) << rb;
    int64_t k_rem = k;
    while (rb > 0) {
        const int w = rb < kDigitBits ? rb : kDigitBits;
        const int shift = rb - w;
        const uint32_t dmask = (1u << w) - 1u;
        const uint64_t want = rb >= 64 ? 0ull : (prefix >> rb);
        const int rbs = rb >= 64 ? 63 : rb;          // shift amount that is always defined
        const bool all = rb >= 64;
        items.for_each([&](uint64_t c) {
            if (all || (c >> rbs) == want) atomicAdd(&sm.hist[(uint32_t)(c >> shift) & dmask], 1u);
        });
        __syncthreads();
        if (wave == 0) {
            // digits in descending order: position p = kBinsPerLane * lane + i <-> bin kBins-1-p
            uint32_t local = 0;
#pragma unroll 8
            for (int i = 0; i < kBinsPerLane; ++i)   // rotated start: lanes hit different LDS banks
                local += sm.hist[kBins - 1 - (kBinsPerLane * lane + ((i + lane) & (kBinsPerLane - 1)))];
            uint32_t incl = local;
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t v = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += v;
            }
            uint32_t run = incl - local;
            if ((int64_t)run < k_rem && k_rem <= (int64_t)incl) {   // exactly one lane
                for (int i = 0; i < kBinsPerLane; ++i) {
                    const int bin = kBins - 1 - (kBinsPerLane * lane + i);
                    const uint32_t c = sm.hist[bin];
                    if ((int64_t)run < k_rem && k_rem <= (int64_t)(run + c)) {
                        sm.bin = (uint32_t)bin;
                        sm.above = run;
                        sm.cb = c;
                    }
                    run += c;
                }
            }
        }
        __syncthreads();
        const uint32_t bin = sm.bin, above = sm.above, cb = sm.cb;
        __syncthreads();
        for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
        prefix |= (uint64_t)bin << shift;
        k_rem -= above;
        rb = shift;
        if ((int64_t)cb == k_rem) break;   // the whole bin is selected
        __syncthreads();
    }
    __syncthreads();
    return prefix;
}

// Slots the selection does not fill: position -1, score -inf.
__device__ __forceinline__ void pad_outputs(int k_eff, int k, int32_t* idx, float* vals) {
    for (int j = k_eff + (int)threadIdx.x; j < k; j += kSelThreads) {
        idx[j] = -1;
        vals[j] = -INFINITY;
    }
}

// Write the items with key >= T (exactly k_eff of them) to idx/vals and pad up to k.
// Order: wave-major, then slot, then lane -- fixed, and each store instruction of a wave
// writes one contiguous run.
template <class It>
__device__ void wg_emit(const It& items, uint64_t T, int k_eff, int k, int32_t* idx, float* vals, SelShared& sm) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t wave_total = 0;
    items.for_each_sync([&](uint64_t c, bool present) { wave_total += (uint32_t)__popcll(__ballot(present && c >= T)); });
    __syncthreads();
    if (lane == 0) sm.wave_tot[wave] = wave_total;
    __syncthreads();
    uint32_t run = 0;
    for (int w = 0; w < wave; ++w) run += sm.wave_tot[w];
    items.for_each_sync([&](uint64_t c, bool present) {
        const bool sel = present && c >= T;
        const uint64_t m = __ballot(sel);
        if (sel) {
            const uint32_t slot = run + (uint32_t)mask_rank(m);
            if (slot < (uint32_t)k_eff) {     // always true; guards the output buffer
                idx[slot] = (int32_t)composite_pos(c);
                vals[slot] = composite_score(c);
            }
        }
        run += (uint32_t)__popcll(m);
    });
    pad_outputs(k_eff, k, idx, vals);
}

// Threshold estimate: the rank-th largest of the sample scores of each head; also clears
// the head's fallback flag for the scan that follows.
__global__ void __launch_bounds__(kSelThreads) threshold_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = prefix_len(bf.len[b], sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    if (N == 0) {                    // nothing to search for this sequence
        if (threadIdx.x == 0) {
            bf.thr[bh] = INFINITY;
            bf.flags[bh] = 0;
            if (bh == 0) *bf.fallback_total = 0;
        }
        return;
    }
    const Plan pl = make_plan(N, k_eff);
    const SrcDense src{bf.samp + bh * sh.samp_cap, (int64_t)pl.n_samp};
    const Items<(kSampMax + kSelThreads - 1) / kSelThreads, SrcDense> items(src);
    uint64_t kmax;
    const int rank = pl.rank < pl.n_samp ? pl.rank : pl.n_samp;
    const uint64_t T = wg_select_kth(items, (int64_t)pl.n_samp, (int64_t)rank, sm, &kmax);
    if (threadIdx.x == 0) {
        bf.thr[bh] = composite_score(T);
        bf.flags[bh] = 0;
        if (bh == 0) *bf.fallback_total = 0;
    }
}

// Exact selection among the candidates the filtered scan kept, read from the interleaved
// per-wave segments.
__global__ void __launch_bounds__(kSelThreads) select_candidates_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = prefix_len(bf.len[b], sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;

    if (k_eff == 0) {                // nothing to search: only padding to write
        pad_outputs(0, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k);
        if (tid == 0) bf.hmax[bh] = -INFINITY;
        return;
    }
    // segment lengths: total, longest
    uint32_t sum = 0, mxl = 0;
    for (int g = tid; g < sh.n_seg; g += kSelThreads) {
        const uint32_t c = bf.seg_cnt[bh * sh.n_seg + g];
        sm.seg_len[g] = c;
        sum += c;
        mxl = c > mxl ? c : mxl;
    }
    for (int o = 32; o > 0; o >>= 1) {
        sum += __shfl_xor(sum, o, kWave);
        const uint32_t t = __shfl_xor(mxl, o, kWave);
        mxl = t > mxl ? t : mxl;
    }
    if (lane == 0) { sm.wave_tot[wave] = sum; sm.red_max[wave] = mxl; }
    __syncthreads();
    uint32_t total = 0, max_len = 0;
    for (int w = 0; w < kSelWaves; ++w) {
        total += sm.wave_tot[w];
        max_len = (uint32_t)sm.red_max[w] > max_len ? (uint32_t)sm.red_max[w] : max_len;
    }
    __syncthreads();
    if (max_len > (uint32_t)sh.seg_cap || total < (uint32_t)k_eff) {   // uniform: a segment overflowed, or
        if (tid == 0) {                                                // the threshold was too high
            bf.flags[bh] = 1;
            atomicAdd(bf.fallback_total, 1u);
        }
        return;
    }
    const SrcSeg src{bf.cand + bh * (int64_t)sh.cand_cap, sm.seg_len, sh.n_seg, (int)max_len};
    const Items<(32768 + kSelThreads - 1) / kSelThreads, SrcSeg> items(src);
    uint64_t kmax;
    const uint64_t T = wg_select_kth(items, (int64_t)total, (int64_t)k_eff, sm, &kmax);
    wg_emit(items, T, k_eff, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k, sm);
    if (tid == 0) bf.hmax[bh] = composite_score(kmax);
}

// Exact selection over the full score row (general path, and heads the filter gave up on).
__global__ void __launch_bounds__(kSelThreads) select_full_kernel(Shape sh, Bufs bf, int only_flagged) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    if (only_flagged && !bf.flags[bh]) return;
    const int64_t N = prefix_len(bf.len[b], sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    if (k_eff == 0) {
        pad_outputs(0, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k);
        if (threadIdx.x == 0) bf.hmax[bh] = -INFINITY;
        return;
    }
    const SrcDense src{bf.scores + bh * sh.Ncap, N};
    const Items<(8192 + kSelThreads - 1) / kSelThreads, SrcDense> items(src);
    uint64_t kmax;
    const uint64_t T = wg_select_kth(items, N, (int64_t)k_eff, sm, &kmax);
    wg_emit(items, T, k_eff, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k, sm);
    if (threadIdx.x == 0) bf.hmax[bh] = composite_score(kmax);
}

hipError_t launch_threshold(const Shape& s, const Bufs& b, hipStream_t st) {
    hipLaunchKernelGGL(threshold_kernel, dim3(s.Hq, s.B), dim3(kSelThreads), 0, st, s, b);
    return hipGetLastError();
}
hipError_t launch_select_candidates(const Shape& s, const Bufs& b, hipStream_t st) {
    hipLaunchKernelGGL(select_candidates_kernel, dim3(s.Hq, s.B), dim3(kSelThreads), 0, st, s, b);
    return hipGetLastError();
}
hipError_t launch_select_full(const Shape& s, const Bufs& b, bool only_flagged, hipStream_t st) {
    hipLaunchKernelGGL(select_full_kernel, dim3(s.Hq, s.B), dim3(kSelThreads), 0, st, s, b, only_flagged ? 1 : 0);
    return hipGetLastError();
}

}  // namespace tka
