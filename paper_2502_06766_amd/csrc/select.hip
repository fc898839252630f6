// Exact top-k selection (the result of the paper's knn_search: the k largest scores
// `vals` and their positions `I`), by radix select on unique 64-bit keys
// (order-preserving image of the fp32 score, then inverted position), so that equal
// scores resolve to the lower position and the selected set never depends on the order
// in which candidates were produced.
#include "device_utils.h"
#include "internal.h"

namespace tka {

struct SelShared {
    uint32_t hist[256];
    uint64_t red_max[kSelThreads / kWave];
    uint64_t red_min[kSelThreads / kWave];
    uint64_t bc_max, bc_min;
    uint32_t bin, above, cb;
    uint32_t out_cnt;
};

// sources of (score, position) items
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

// Returns T such that exactly k of the n items have key >= T (1 <= k <= n).
// *kmax receives the largest key.  All threads of the workgroup must call it.
template <class Src>
__device__ uint64_t wg_select_kth(const Src& src, int64_t n, int64_t k, SelShared& sm, uint64_t* kmax) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int nwave = blockDim.x >> 6;
    // range of the keys
    uint64_t mx = 0, mn = ~0ull;
    for (int64_t i = tid; i < n; i += blockDim.x) {
        const uint64_t c = src.key(i);
        mx = c > mx ? c : mx;
        mn = c < mn ? c : mn;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t a = __shfl_xor(mx, o, 64), b = __shfl_xor(mn, o, 64);
        mx = a > mx ? a : mx;
        mn = b < mn ? b : mn;
    }
    if (lane == 0) { sm.red_max[wave] = mx; sm.red_min[wave] = mn; }
    for (int i = tid; i < 256; i += blockDim.x) sm.hist[i] = 0;
    __syncthreads();
    if (tid == 0) {
        for (int w = 0; w < nwave; ++w) {
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
    int rb = 64 - __clzll((long long)(mx ^ mn));   // mx != mn here because keys are unique and n >= 2
    uint64_t prefix = rb >= 64 ? 0ull : (mx >> rb) << rb;
    int64_t k_rem = k;
    while (rb > 0) {
        const int w = rb < 8 ? rb : 8;
        const int shift = rb - w;
        const uint32_t dmask = (1u << w) - 1u;
        for (int64_t i = tid; i < n; i += blockDim.x) {
            const uint64_t c = src.key(i);
            const bool match = rb >= 64 ? true : ((c >> rb) == (prefix >> rb));
            if (match) atomicAdd(&sm.hist[(uint32_t)(c >> shift) & dmask], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // position p = 4 lane + i (descending digit order) <-> bin 255 - p
            uint32_t c4[4], local = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c4[i] = sm.hist[255 - (4 * lane + i)]; local += c4[i]; }
            uint32_t incl = local;
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t v = __shfl_up(incl, o, 64);
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
        for (int i = tid; i < 256; i += blockDim.x) sm.hist[i] = 0;
        prefix |= (uint64_t)bin << shift;
        k_rem -= above;
        rb = shift;
        if ((int64_t)cb == k_rem) break;   // the whole bin is selected
        __syncthreads();
    }
    __syncthreads();
    return prefix;
}

// Write the items with key >= T (exactly k_eff of them) to idx/vals, pad up to k.
template <class Src>
__device__ void wg_emit(const Src& src, int64_t n, uint64_t T, int k_eff, int k, int32_t* idx, float* vals,
                        SelShared& sm) {
    const int tid = threadIdx.x, lane = lane_id();
    if (tid == 0) sm.out_cnt = 0;
    __syncthreads();
    const int64_t n_round = (n + blockDim.x - 1) / blockDim.x * blockDim.x;
    for (int64_t i = tid; i < n_round; i += blockDim.x) {
        uint64_t c = 0;
        bool sel = false;
        if (i < n) { c = src.key(i); sel = c >= T; }
        const uint64_t m = __ballot(sel);
        if (m) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&sm.out_cnt, (uint32_t)__popcll(m));
            base = wave_first_u32(base);
            if (sel) {
                const uint32_t slot = base + (uint32_t)mask_rank(m);
                if (slot < (uint32_t)k_eff) {     // always true; guards the output buffer
                    idx[slot] = (int32_t)composite_pos(c);
                    vals[slot] = composite_score(c);
                }
            }
        }
    }
    for (int j = k_eff + tid; j < k; j += blockDim.x) {
        idx[j] = -1;
        vals[j] = -INFINITY;
    }
}

// Threshold estimate: the rank-th largest of the sample scores of each head; also clears
// the head's candidate counter and fallback flag for the scan that follows.
__global__ void __launch_bounds__(kSelThreads) threshold_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const Plan pl = make_plan(N, k_eff);
    SrcDense src{bf.samp + bh * sh.samp_cap};
    uint64_t kmax;
    int rank = pl.rank < pl.n_samp ? pl.rank : pl.n_samp;
    const uint64_t T = wg_select_kth(src, pl.n_samp, rank, sm, &kmax);
    if (threadIdx.x == 0) {
        bf.thr[bh] = composite_score(T);
        bf.cand_cnt[bh] = 0;
        bf.flags[bh] = 0;
        if (bh == 0) *bf.fallback_total = 0;
    }
}

// Exact selection among the candidates the filtered scan kept.
__global__ void __launch_bounds__(kSelThreads) select_candidates_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const uint32_t cnt = bf.cand_cnt[bh];
    if (cnt < (uint32_t)k_eff || cnt > (uint32_t)sh.cand_cap) {
        if (threadIdx.x == 0) {
            bf.flags[bh] = 1;
            atomicAdd(bf.fallback_total, 1u);
        }
        return;
    }
    SrcCand src{bf.cand + bh * (int64_t)sh.cand_cap};
    uint64_t kmax;
    const uint64_t T = wg_select_kth(src, (int64_t)cnt, (int64_t)k_eff, sm, &kmax);
    wg_emit(src, (int64_t)cnt, T, k_eff, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k, sm);
    if (threadIdx.x == 0) bf.hmax[bh] = composite_score(kmax);
}

// Exact selection over the full score row (general path, and heads the filter gave up on).
__global__ void __launch_bounds__(kSelThreads) select_full_kernel(Shape sh, Bufs bf, int only_flagged) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    if (only_flagged && !bf.flags[bh]) return;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    SrcDense src{bf.scores + bh * sh.Ncap};
    uint64_t kmax;
    const uint64_t T = wg_select_kth(src, N, (int64_t)k_eff, sm, &kmax);
    wg_emit(src, N, T, k_eff, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k, sm);
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
