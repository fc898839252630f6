// Exact top-k selection (the result of the paper's knn_search: the k largest scores
// `vals` and their positions `I`), by radix select on unique 64-bit keys
// (order-preserving image of the fp32 score, then inverted position), so that equal
// scores resolve to the lower position and the selected set never depends on the order
// in which candidates were produced.  One workgroup of 1024 threads per (sequence, head).
//
// The first CPT * 1024 items of a head are held in registers for all passes; anything
// beyond is re-read from memory in batches of independent loads.  Output order is fixed
// (thread-major), so repeated calls return bit-identical results.
#include "device_utils.h"
#include "internal.h"

namespace tka {

constexpr int kSelWaves = kSelThreads / kWave;

struct SelShared {
    uint32_t hist[256];
    uint64_t red_max[kSelWaves];
    uint64_t red_min[kSelWaves];
    uint64_t bc_max, bc_min;
    uint32_t bin, above, cb;
    uint32_t wave_tot[kSelWaves];
    uint32_t scan_total;
    uint32_t seg_off[kMaxSeg];
    uint32_t seg_len[kMaxSeg];
};

// sources of (score, position) items; key 0 never occurs for a real item (it would need
// the score bit pattern 0xFFFFFFFF, a NaN) and marks an empty register slot
struct SrcDense {            // scores[i], position i
    const float* s;
    __device__ __forceinline__ uint64_t key(int64_t i) const { return composite(s[i], (uint32_t)i); }
};
struct SrcCand {             // packed (score bits << 32 | position)
    const uint64_t* c;
    __device__ __forceinline__ uint64_t key(int64_t i) const {
        const uint64_t e = c[i];
        return composite(__uint_as_float((uint32_t)(e >> 32)), (uint32_t)e);
    }
};

// The items of one head as seen by one thread: register slots j hold item j * 1024 + tid,
// the tail [CPT * 1024, n) is streamed.
template <int CPT, class Src>
struct Items {
    uint64_t kc[CPT > 0 ? CPT : 1];
    const Src& src;
    const int64_t n;
    __device__ __forceinline__ Items(const Src& s, int64_t n_) : src(s), n(n_) {
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int64_t i = (int64_t)j * kSelThreads + threadIdx.x;
            kc[j] = i < n ? src.key(i) : 0ull;
        }
    }
    template <class F>
    __device__ __forceinline__ void for_each(F f) const {
#pragma unroll
        for (int j = 0; j < CPT; ++j)
            if (kc[j]) f(kc[j]);
        constexpr int U = 8;
        for (int64_t base = (int64_t)CPT * kSelThreads + threadIdx.x; base < n; base += (int64_t)U * kSelThreads) {
            uint64_t t[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = base + (int64_t)u * kSelThreads;
                t[u] = i < n ? src.key(i) : 0ull;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (t[u]) f(t[u]);
        }
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
    for (int i = tid; i < 256; i += kSelThreads) sm.hist[i] = 0;
    __syncthreads();
    if (tid == 0) {
        for (int w = 0; w < kSelWaves; ++w) {
            mx = sm.red_max[w] > mx ? sm.red_max[w] : mx;
            mn = sm.red_min[w] < mn ? sm.red_min[w] : mn;
        }
        sm.bc_max = mx; sm.bc_min = mn;
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
        const int w = rb < 8 ? rb : 8;
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
            // position p = 4 lane + i (descending digit order) <-> bin 255 - p
            uint32_t c4[4], local = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c4[i] = sm.hist[255 - (4 * lane + i)]; local += c4[i]; }
            uint32_t incl = local;
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t v = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += v;
            }
            uint32_t run = incl - local;
            if ((int64_t)run < k_rem && k_rem <= (int64_t)incl) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if ((int64_t)run < k_rem && k_rem <= (int64_t)(run + c4[i])) {
                        sm.bin = 255 - (4 * lane + i);
                        sm.above = run;
                        sm.cb = c4[i];
                    }
                    run += c4[i];
                }
            }
        }
        __syncthreads();
        const uint32_t bin = sm.bin, above = sm.above, cb = sm.cb;
        __syncthreads();
        for (int i = tid; i < 256; i += kSelThreads) sm.hist[i] = 0;
        prefix |= (uint64_t)bin << shift;
        k_rem -= above;
        rb = shift;
        if ((int64_t)cb == k_rem) break;   // the whole bin is selected
        __syncthreads();
    }
    __syncthreads();
    return prefix;
}

// Write the items with key >= T (exactly k_eff of them) to idx/vals in thread-major
// order, pad up to k.
template <class It>
__device__ void wg_emit(const It& items, uint64_t T, int k_eff, int k, int32_t* idx, float* vals, SelShared& sm) {
    uint32_t mine = 0;
    items.for_each([&](uint64_t c) { mine += c >= T ? 1u : 0u; });
    uint32_t total;
    uint32_t off = wg_exclusive_scan(mine, sm, &total);
    items.for_each([&](uint64_t c) {
        if (c >= T) {
            if (off < (uint32_t)k_eff) {     // always true; guards the output buffer
                idx[off] = (int32_t)composite_pos(c);
                vals[off] = composite_score(c);
            }
            ++off;
        }
    });
    for (int j = k_eff + (int)threadIdx.x; j < k; j += kSelThreads) {
        idx[j] = -1;
        vals[j] = -INFINITY;
    }
}

// Threshold estimate: the rank-th largest of the sample scores of each head; also clears
// the head's fallback flag for the scan that follows.
__global__ void __launch_bounds__(kSelThreads) threshold_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const Plan pl = make_plan(N, k_eff);
    const SrcDense src{bf.samp + bh * sh.samp_cap};
    const Items<kSampMax / kSelThreads, SrcDense> items(src, pl.n_samp);
    uint64_t kmax;
    const int rank = pl.rank < pl.n_samp ? pl.rank : pl.n_samp;
    const uint64_t T = wg_select_kth(items, (int64_t)pl.n_samp, (int64_t)rank, sm, &kmax);
    if (threadIdx.x == 0) {
        bf.thr[bh] = composite_score(T);
        bf.flags[bh] = 0;
        if (bh == 0) *bf.fallback_total = 0;
    }
}

// Exact selection among the candidates the filtered scan kept: pack the head's segments
// into one list, then select among them.
__global__ void __launch_bounds__(kSelThreads) select_candidates_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;

    uint32_t c = tid < sh.n_seg ? bf.seg_cnt[bh * sh.n_seg + tid] : 0u;
    const uint32_t over = __syncthreads_or(c > (uint32_t)sh.seg_cap ? 1 : 0);
    uint32_t total;
    const uint32_t off = wg_exclusive_scan(c, sm, &total);
    if (over || total < (uint32_t)k_eff) {      // uniform: a segment overflowed, or the threshold was too high
        if (tid == 0) {
            bf.flags[bh] = 1;
            atomicAdd(bf.fallback_total, 1u);
        }
        return;
    }
    if (tid < sh.n_seg) { sm.seg_off[tid] = off; sm.seg_len[tid] = c; }
    __syncthreads();
    const uint64_t* segs = bf.cand + bh * (int64_t)sh.cand_cap;
    uint64_t* flat = bf.cand_flat + bh * (int64_t)sh.cand_cap;
    for (int s = wave; s < sh.n_seg; s += kSelWaves) {
        const uint32_t len = sm.seg_len[s], o0 = sm.seg_off[s];
        for (uint32_t o = lane; o < len; o += kWave) flat[o0 + o] = segs[(int64_t)s * sh.seg_cap + o];
    }
    __syncthreads();    // the packed list is read back by other waves of this workgroup

    const SrcCand src{flat};
    const Items<32, SrcCand> items(src, (int64_t)total);
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
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const SrcDense src{bf.scores + bh * sh.Ncap};
    const Items<8, SrcDense> items(src, N);
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
