// Workgroup-level building blocks of the exact top-k selection (radix select over
// order-preserving score keys, position tie-break, fixed-order emission), shared by the
// selection kernels (select.hip) and the tail of the filtered path (tail.hip).
#pragma once
#include "device_utils.h"
#include "internal.h"

namespace tka {

constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kDigitBits = 9;                  // radix digit width (the best of 8..11 measured)
constexpr int kBins = 1 << kDigitBits;
constexpr int kBinsPerLane = kBins / kWave;

struct SelShared {
    uint32_t hist[kBins];
    uint32_t red_max[kSelWaves];
    uint32_t red_min[kSelWaves];
    uint32_t bc_max, bc_min;
    uint32_t bin, above, cb;
    uint32_t wave_tot[kSelWaves];
};

// Order-preserving key of a score (-0 counts as +0).  0 would need the bit pattern of a
// NaN, so 0 marks "no item"; inverted positions 0xFFFFFFFF - p are >= 2^31 and never 0.
__device__ __forceinline__ uint32_t score_key(float s) { return ord_from_bits(__float_as_uint(s + 0.0f)); }
__device__ __forceinline__ float key_score(uint32_t o) { return __uint_as_float(bits_from_ord(o)); }

// ---------------------------------------------------------------------------------------
// Sources: slot i of a head either holds an item (score, position) or is empty.
// ---------------------------------------------------------------------------------------
template <int NT>            // NT: threads of the workgroup
struct SrcDenseT {           // scores[i] at position i, i < n
    static constexpr int kThreads = NT;
    const float* s;
    int64_t n;
    typedef float raw_t;
    __device__ __forceinline__ int64_t slots() const { return n; }
    __device__ __forceinline__ bool valid(int64_t i) const { return i < n; }
    __device__ __forceinline__ const float* where(int64_t i) const { return s + i; }
    __device__ __forceinline__ uint32_t key(float r) const { return score_key(r); }
    __device__ __forceinline__ uint32_t ipos(float, int64_t i) const { return 0xFFFFFFFFu - (uint32_t)i; }
    // the position of a cached slot is implied by the slot
    __device__ __forceinline__ void stash(int, float) const {}
    __device__ __forceinline__ uint32_t cached_ipos(int j) const {
        return 0xFFFFFFFFu - (uint32_t)(j * NT + (int)threadIdx.x);
    }
};
// The items of one head as seen by one thread: register slot j holds the score key of
// source slot j * kSelThreads + tid, later slots are streamed.  Every lane of a wave
// visits the same slots in the same order (with a per-lane "present" flag), so visitors
// may use wave-wide ballots.
template <int CPT, class Src>
struct Items {
    static constexpr int kThreads = Src::kThreads;
    uint32_t kc[CPT > 0 ? CPT : 1];
    const Src src;      // by value: keeps the LDS pointers inside visible to the compiler as LDS
    __device__ __forceinline__ Items(const Src& s) : src(s) {
        constexpr int BMAX = 16;                                   // independent loads per batch
        constexpr int B = CPT < BMAX ? (CPT > 0 ? CPT : 1) : BMAX;
#pragma unroll
        for (int j0 = 0; j0 < CPT; j0 += B) {
            typename Src::raw_t r[B];
            bool ok[B];
#pragma unroll
            for (int u = 0; u < B; ++u) {
                if (j0 + u < CPT) {          // CPT need not be a multiple of the batch
                    const int64_t i = (int64_t)(j0 + u) * kThreads + threadIdx.x;
                    ok[u] = src.valid(i);
                    r[u] = *src.where(ok[u] ? i : 0);
                }
            }
#pragma unroll
            for (int u = 0; u < B; ++u) {
                if (j0 + u < CPT) {
                    kc[j0 + u] = ok[u] ? src.key(r[u]) : 0u;
                    if (ok[u]) src.stash(j0 + u, r[u]);
                }
            }
        }
    }
    // f(score key, inverted position, present) for every slot, all lanes in lock step
    template <class F>
    __device__ __forceinline__ void visit(F f) const {
#pragma unroll
        for (int j = 0; j < CPT; ++j) f(kc[j], src.cached_ipos(j), kc[j] != 0u);
        constexpr int U = 8;
        const int64_t n_slots = src.slots();
        for (int64_t base = (int64_t)CPT * kThreads; base < n_slots; base += (int64_t)U * kThreads) {
            typename Src::raw_t r[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
                ok[u] = src.valid(i);
                r[u] = *src.where(ok[u] ? i : 0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
                f(ok[u] ? src.key(r[u]) : 0u, src.ipos(r[u], i), ok[u]);
            }
        }
    }
};

// Result of a radix select of the k largest among a multiset of 32-bit keys: the wanted
// keys are all keys > T plus `need` of the `have` keys in the threshold class.  The class
// is "key == T" when `exact`; otherwise the select stopped early because the whole last
// bin was wanted (need == have) and the wanted keys are simply all keys >= T.
struct Sel32 {
    uint32_t T, kmax, need, have;
    bool exact;
};

// `keys(f)` must call f(key, present) for every slot, slot-synchronously.
// 1 <= k <= number of present keys.  All threads of the workgroup must call it.
// With `bounded`, the caller already knows the largest key `hi` and a lower bound `lo` of
// all keys, and the pass that would find them is skipped.  `max_passes` > 0 stops the
// refinement early: the result then has need <= have and T is only a lower bound of the
// k-th key (for callers that can live with a few extra keys at or above T).
template <int NT, class Keys>     // NT: threads of the workgroup
__device__ __forceinline__ Sel32 wg_select32(Keys keys, int64_t k, SelShared& sm, bool bounded = false,
                                             uint32_t lo = 0u, uint32_t hi = 0u, int max_passes = 0) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    uint32_t mx = hi, mn = lo;
    if (!bounded) {
        mx = 0u; mn = ~0u;
        keys([&](uint32_t c, bool present) {
            if (present) {
                mx = c > mx ? c : mx;
                mn = c < mn ? c : mn;
            }
        });
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t a = __shfl_xor(mx, o, kWave), b = __shfl_xor(mn, o, kWave);
            mx = a > mx ? a : mx;
            mn = b < mn ? b : mn;
        }
    }
    __syncthreads();                  // the shared scratch may still be read by a previous select
    if (!bounded && lane == 0) { sm.red_max[wave] = mx; sm.red_min[wave] = mn; }
    for (int i = tid; i < kBins; i += NT) sm.hist[i] = 0;
    __syncthreads();
    if (!bounded) {
        if (wave == 0) {
            mx = lane < (NT / kWave) ? sm.red_max[lane] : 0u;
            mn = lane < (NT / kWave) ? sm.red_min[lane] : ~0u;
            for (int o = 32; o > 0; o >>= 1) {
                const uint32_t a = __shfl_xor(mx, o, kWave), b = __shfl_xor(mn, o, kWave);
                mx = a > mx ? a : mx;
                mn = b < mn ? b : mn;
            }
            if (lane == 0) { sm.bc_max = mx; sm.bc_min = mn; }
        }
        __syncthreads();
        mx = sm.bc_max; mn = sm.bc_min;
    }
    Sel32 res;
    res.kmax = mx;
    if (mx == mn) {                   // one distinct key: the class is everything
        uint32_t cnt = 0;
        keys([&](uint32_t, bool present) { cnt += (uint32_t)__popcll(__ballot(present)); });
        __syncthreads();
        if (lane == 0) sm.wave_tot[wave] = cnt;
        __syncthreads();
        uint32_t total = 0;
        for (int w = 0; w < (NT / kWave); ++w) total += sm.wave_tot[w];
        res.T = mx; res.need = (uint32_t)k; res.have = total; res.exact = true;
        return res;
    }
    // bits above `rb` are common to every remaining key and fixed in `prefix`
    int rb = 32 - __clz((int)(mx ^ mn));
    uint32_t prefix = rb >= 32 ? 0u : (mx >> rb) << rb;
    int64_t k_rem = k;
    uint32_t cb = 0;
    int passes = 0;
    while (true) {
        const int w = rb < kDigitBits ? rb : kDigitBits;
        const int shift = rb - w;
        const uint32_t dmask = (1u << w) - 1u;
        const uint32_t want = rb >= 32 ? 0u : (prefix >> rb);
        const int rbs = rb >= 32 ? 31 : rb;          // a shift amount that is always defined
        const bool all = rb >= 32;
        keys([&](uint32_t c, bool present) {
            if (present && (all || (c >> rbs) == want)) atomicAdd(&sm.hist[(c >> shift) & dmask], 1u);
        });
        __syncthreads();
        if (wave == 0) {
            // digits in descending order: position p = kBinsPerLane * lane + i <-> bin kBins-1-p
            uint32_t local = 0;
#pragma unroll
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
        const uint32_t bin = sm.bin, above = sm.above;
        cb = sm.cb;
        __syncthreads();
        for (int i = tid; i < kBins; i += NT) sm.hist[i] = 0;
        prefix |= bin << shift;
        k_rem -= above;
        rb = shift;
        ++passes;
        if ((int64_t)cb == k_rem || rb == 0) break;   // the whole bin is wanted, or all bits are fixed
        if (passes == max_passes) break;              // good enough for the caller: everything >= prefix
        __syncthreads();
    }
    __syncthreads();
    res.T = prefix;
    res.need = (uint32_t)k_rem;
    res.have = cb;
    res.exact = rb == 0;          // false also after an early stop: T = prefix <= the k-th key
    return res;
}

// Slots the selection does not fill: position -1, score -inf.
__device__ __forceinline__ void pad_outputs(int k_eff, int k, int32_t* idx, float* vals) {
    for (int j = k_eff + (int)threadIdx.x; j < k; j += (int)blockDim.x) {
        idx[j] = -1;
        vals[j] = -INFINITY;
    }
}

// Exact top-k_eff of the items: select on the score keys, break a tie at the k-th score
// by position, write idx/vals (wave-major, then slot, then lane: fixed, and every store
// instruction of a wave writes one contiguous run) and pad up to k.  Returns the largest key.
template <class It>
__device__ __forceinline__ uint32_t wg_topk_emit(const It& items, int k_eff, int k, int32_t* idx, float* vals,
                                                 SelShared& sm, bool bounded = false, uint32_t lo = 0u,
                                                 uint32_t hi = 0u) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const Sel32 s = wg_select32<It::kThreads>([&](auto f) { items.visit([&](uint32_t c, uint32_t, bool p) { f(c, p); }); },
                                (int64_t)k_eff, sm, bounded, lo, hi);
    const bool ties = s.need < s.have;    // (uniform) more items share the k-th score than fit
    uint32_t T2 = 0u;                     // then: inverted-position threshold inside the class key == T
    if (ties) {
        // positions are unique, so this select always ends with need == have: ipos >= T2 is exact
        const Sel32 t = wg_select32<It::kThreads>(
            [&](auto f) { items.visit([&](uint32_t c, uint32_t ip, bool p) { f(ip, p && c == s.T); }); },
            (int64_t)s.need, sm);
        T2 = t.T;
    }
    auto wanted = [&](uint32_t c, uint32_t ip, bool present) {
        return present && (c > s.T || (c == s.T && (!ties || ip >= T2)));
    };
    uint32_t wave_total = 0;
    if (ties) {
        items.visit([&](uint32_t c, uint32_t ip, bool p) {
            wave_total += (uint32_t)__popcll(__ballot(wanted(c, ip, p)));
        });
    } else {       // the score alone decides: no need to fetch the positions for counting
        items.visit([&](uint32_t c, uint32_t, bool p) {
            wave_total += (uint32_t)__popcll(__ballot(p && c >= s.T));
        });
    }
    __syncthreads();
    if (lane == 0) sm.wave_tot[wave] = wave_total;
    __syncthreads();
    uint32_t run = 0;
    for (int w = 0; w < wave; ++w) run += sm.wave_tot[w];
    items.visit([&](uint32_t c, uint32_t ip, bool p) {
        const bool sel = wanted(c, ip, p);
        const uint64_t m = __ballot(sel);
        if (sel) {
            const uint32_t slot = run + (uint32_t)mask_rank(m);
            if (slot < (uint32_t)k_eff) {     // always true; guards the output buffer
                idx[slot] = (int32_t)(0xFFFFFFFFu - ip);
                vals[slot] = key_score(c);
            }
        }
        run += (uint32_t)__popcll(m);
    });
    pad_outputs(k_eff, k, idx, vals);
    return s.kmax;
}

// Exact selection of one head over its full score row (the general path's selection).
template <int NT, int CPT>     // the first CPT * NT scores stay in registers, the rest is streamed
__device__ __forceinline__ uint32_t wg_select_dense(const Shape& sh, const Bufs& bf, int64_t bh, int64_t N, int k_eff,
                                                    SelShared& sm) {
    const SrcDenseT<NT> src{bf.scores + bh * sh.Ncap, N};
    const Items<CPT, SrcDenseT<NT>> items(src);
    const uint32_t kmax = wg_topk_emit(items, k_eff, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k, sm);
    if (threadIdx.x == 0) bf.hmax[bh] = key_score(kmax);
    return kmax;              // key of the largest score (uniform)
}

}  // namespace tka
