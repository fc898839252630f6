// Exact top-k selection (the result of the paper's knn_search: the k largest scores
// `vals` and their positions `I`), by radix select.  Scores are compared through an
// order-preserving 32-bit image of the fp32 value; when the k-th score is shared by more
// items than fit, a second radix select over the (unique) inverted positions of those
// items picks the lowest positions, so equal scores resolve to the lower position and the
// selected set never depends on the order in which candidates were produced.
// One workgroup per (sequence, head).
//
// The first CPT * kSelThreads items of a head keep their score key in registers for all
// passes (and, for candidate lists, their position in LDS); anything beyond is re-read
// from memory in batches of independent loads.  Output order is fixed (wave-major), so
// repeated calls return bit-identical results.
#include "device_utils.h"
#include "internal.h"
#include "select_common.h"

namespace tka {

// Threshold estimate of each head: a score with about `rank` of the head's sample scores at or above it,
// by linear binning between the smallest and the largest sample (512 bins): the threshold is
// the lower edge of the bin that holds the rank-th largest sample.  The handful of samples of
// that bin below the rank-th only make the candidate list a little longer (the threshold is a
// heuristic to begin with: the tail checks the candidate count and redoes a head exactly when the
// list does not hold its k best keys).  (A radix select over the float bit pattern spends its
// first digit on sign and exponent, where a few bins take nearly all samples: thousands of
// shared-memory atomics on half a dozen addresses.)  The same histogram gives the parameters of
// tail_bin(), which the tail of the filtered path uses to sort candidates coarsely by score.
// When the range of the samples is so wide that only a few bins lie between the threshold and the
// top of the band the k-th score is expected in, the samples of those bins are binned once more.
// Also clears the head's fallback flag.
constexpr int kThrRefineBelow = 8;   // the bins between threshold and band top are binned again when fewer than this
template <int CPT, int NT>     // NT threads; the launcher makes sure n_samp <= CPT * NT <= samp_cap
__global__ void __launch_bounds__(NT) threshold_kernel(Shape sh, Bufs bf) {
    constexpr int NB = 512, NW = NT / kWave, BPL = NB / kWave;
    __shared__ uint32_t hist[NB];
    __shared__ float red_mx[NW], red_mn[NW];
    __shared__ uint32_t s_bin[4];
    const int b = blockIdx.y, h = blockIdx.x;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    // the sample scores are asked for before the sample size is known (it depends on the sequence
    // length, another trip to memory); what lies beyond the sample is ignored below
    const float* samp = bf.samp + bh * sh.samp_cap;
    float sv[CPT];
#pragma unroll
    for (int j = 0; j < CPT; ++j) sv[j] = samp[j * NT + tid];
    for (int i = tid; i < NB; i += NT) hist[i] = 0;
    auto leave = [&](float thr, uint32_t flag, float bin_lo, float bin_inv) {
        if (tid == 0) {
            bf.thr[bh] = thr;
            bf.bins[2 * bh] = bin_lo;
            bf.bins[2 * bh + 1] = bin_inv;
            bf.flags[bh] = flag;
            if (bh == 0) *bf.fallback_total = 0;
        }
    };
    if (prefix_len(visible_len(sh, bf, b), sh.window) == 0) {   // nothing to search for this sequence
        leave(INFINITY, 0u, 0.f, 0.f);
        return;
    }
    // the sample was drawn by the plan of the cache sequence (shared by all its queries)
    const int64_t N = prefix_len(bf.len[cache_seq(sh, b)], sh.window);
    const Plan pl = make_plan(N, sh.k < N ? sh.k : (int)N, sh.indexed);
    // A sequence of the batch for which the filter is not worth it (a few tokens only, or k so dense that the
    // candidate list cannot hold what passes) gets its threshold like any other: the scan still counts what
    // reaches it per bin even where the list overflows, and the tail sorts the keys by those counts.  Its
    // heads are marked so that they are not reported as fallbacks (bit 0); bit 2 makes the tail ignore a
    // usable list (measurement aid).
    const uint32_t mark = (plan_is_fast(pl, N, sh.cand_cap, true) ? 0u : 1u) | (sh.force_redo ? 4u : 0u);
    const int n_samp = pl.n_samp;
    const uint32_t rank = (uint32_t)(pl.rank < n_samp ? pl.rank : n_samp);
    const uint32_t rank_lo = (uint32_t)(pl.rank_lo < (int)rank ? pl.rank_lo : (int)rank);
    const uint32_t rank_hi = (uint32_t)(pl.rank_hi < (int)rank_lo ? pl.rank_hi : (int)rank_lo);
    // range of the finite samples (a sample beyond a query's own visible prefix is -inf)
    float mx = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
        const bool ok = j * NT + tid < n_samp;
        if (ok) mx = fmaxf(mx, sv[j]);
        if (ok && sv[j] > -INFINITY) mn = fminf(mn, sv[j]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        mx = fmaxf(mx, wave_xor(mx, o));
        mn = fminf(mn, wave_xor(mn, o));
    }
    if (lane == 0) { red_mx[wave] = mx; red_mn[wave] = mn; }
    __syncthreads();
    mx = red_mx[0]; mn = red_mn[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) { mx = fmaxf(mx, red_mx[w]); mn = fminf(mn, red_mn[w]); }
    // sc1 = 0 puts every sample into bin 0 (all samples equal, none finite, or a range beyond fp32)
    const float range = mx - mn;
    const float sc1 = (range > 0.f && range < INFINITY) ? (float)NB / range : 0.f;
    auto coarse_bin = [&](float v) {
        int bb = 0;
        if (v > -INFINITY) {
            bb = (int)fminf((v - mn) * sc1, (float)(NB - 1));
            bb = bb < 0 ? 0 : bb;
        }
        return bb;
    };
#pragma unroll
    for (int j = 0; j < CPT; ++j)
        if (j * NT + tid < n_samp) atomicAdd(&hist[coarse_bin(sv[j])], 1u);
    __syncthreads();
    // wave 0 walks the bins from the top: the bins in which the count (on top of `above` samples that lie
    // beyond the last bin) reaches each of the three ranks; s_bin[3]: samples above the bin of the smallest rank
    auto walk = [&](uint32_t above) {
        uint32_t c[BPL], local = 0;
#pragma unroll
        for (int i = 0; i < BPL; ++i) {     // lane l owns bins NB - 1 - BPL l - i; rotated start: lanes hit different LDS banks
            const int ii = (i + lane) & (BPL - 1);
            c[i] = hist[NB - 1 - (BPL * lane + ii)];
        }
#pragma unroll
        for (int i = 0; i < BPL; ++i) local += c[i];
        uint32_t incl = local;
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t v = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += v;
        }
        incl += above;
        const uint32_t want[3] = {rank, rank_lo, rank_hi};
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            if (incl - local < want[q] && want[q] <= incl) {   // exactly one lane
                uint32_t run = incl - local;
                int found = 0;
                uint32_t before = run;
#pragma unroll
                for (int i = 0; i < BPL; ++i) {                // bins in descending order: c[] is rotated by the lane
                    uint32_t ci = 0;
#pragma unroll
                    for (int r = 0; r < BPL; ++r) ci = ((r + lane) & (BPL - 1)) == i ? c[r] : ci;
                    if (run < want[q] && want[q] <= run + ci) { found = NB - 1 - (BPL * lane + i); before = run; }
                    run += ci;
                }
                s_bin[q] = (uint32_t)found;
                if (q == 2) s_bin[3] = before;
            }
        }
    };
    if (wave == 0) walk(0u);
    __syncthreads();
    int b1 = (int)s_bin[0], b_lo = (int)s_bin[1], b_hi = (int)s_bin[2];
    // threshold: the lower edge of bin b1.  tail_bin(): fine bins over the band of scores the sample puts the
    // k-th score in, from the lower edge of the bin of sample rank_lo to the upper edge of that of sample rank_hi
    float lo = mn, sc = sc1;
    // A few samples far from the rest (keys every query attends to, say) stretch the range, and the whole band
    // falls into a handful of wide bins: the threshold, a bin's lower edge, then lets several times the wanted
    // candidates through.  The samples of those bins are then binned once more over the bins' own range.
    if (sc1 > 0.f && b_hi - b1 < kThrRefineBelow) {
        const float lo2 = mn + (float)b1 / sc1, hi2 = mn + (float)(b_hi + 1) / sc1;
        const float range2 = hi2 - lo2;
        const float sc2 = range2 > 0.f ? (float)NB / range2 : 0.f;
        const uint32_t above = s_bin[3];                        // samples in the bins above b_hi
        if (sc2 > 0.f && sc2 < INFINITY) {
            __syncthreads();                                    // (everyone has read s_bin)
            for (int i = tid; i < NB; i += NT) hist[i] = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < CPT; ++j) {
                if (j * NT + tid < n_samp) {
                    const int bb = coarse_bin(sv[j]);            // which samples take part is decided as before, bin by bin
                    if (bb >= b1 && bb <= b_hi) {
                        int fb = (int)fminf((sv[j] - lo2) * sc2, (float)(NB - 1));
                        atomicAdd(&hist[fb < 0 ? 0 : fb], 1u);
                    }
                }
            }
            __syncthreads();
            if (wave == 0) walk(above);
            __syncthreads();
            b1 = (int)s_bin[0]; b_lo = (int)s_bin[1]; b_hi = (int)s_bin[2];
            lo = lo2; sc = sc2;
        }
    }
    float thr = mn, bin_lo = mn, bin_inv = 0.f;
    if (sc > 0.f) {
        thr = (b1 == 0 && lo == mn) ? mn : lo + (float)b1 / sc;
        bin_lo = lo + (float)b_lo / sc;
        const float inv = (float)(kTailBins - 2) * sc / (float)(b_hi + 1 - b_lo);
        bin_inv = inv < INFINITY ? inv : 0.f;
    }
    // (a bin-0 threshold must let -inf samples through when the rank reaches that deep: no finite sample is left out)
    if (b1 == 0 && mn == INFINITY) thr = -INFINITY;
    leave(thr, mark, bin_lo, bin_inv);
}

// Exact selection over the full score row, already in the score buffer (general path).
// NT threads per head: a batch of many short sequences is thousands of heads of a few
// thousand scores each, and a workgroup no larger than the row needs keeps more heads in
// flight per compute unit and makes every barrier of the select cheaper.
template <int NT, int CPT>
__global__ void __launch_bounds__(NT) select_full_kernel(Shape sh, Bufs bf) {
    __shared__ SelShared sm;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t N = prefix_len(visible_len(sh, bf, b), sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    if (k_eff == 0) {
        pad_outputs(0, sh.k, bf.sel_idx + bh * sh.k, bf.sel_val + bh * sh.k);
        if (threadIdx.x == 0) bf.hmax[bh] = -INFINITY;
        return;
    }
    wg_select_dense<NT, CPT>(sh, bf, bh, N, k_eff, sm);
}


// The kernel is correct for any register-cache size (what does not fit is streamed); a
// cache much larger than the data only costs loop trips over empty slots, which matters
// when the whole step is a few tens of microseconds.
// A call with many heads (a batch, 512 heads or more) whose rows are small takes 256-thread workgroups: several
// fit a compute unit at once and every barrier of the select is cheaper; one head alone is
// served faster by 1024 threads.
static bool many_small_heads(const Shape& s) { return (int64_t)s.Hq * s.B >= 512; }

hipError_t launch_threshold(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st) {
    const int n_samp = make_plan(Nmax, s.k < Nmax ? s.k : (int)Nmax, s.indexed).n_samp;
    const dim3 grid(s.Hq, s.B);
    static_assert(kSampMax <= 32 * 256, "the threshold kernel keeps every sample score in registers");
    // four waves per head whatever the sample size: the kernel is a chain of short phases between
    // barriers, which cost more with sixteen waves than the longer per-thread loops do with four
#define TKA_TH(CPT_, NT_) hipLaunchKernelGGL((threshold_kernel<CPT_, NT_>), grid, dim3(NT_), 0, st, s, b)
    if (n_samp <= 1024) TKA_TH(4, 256);
    else if (n_samp <= 2048) TKA_TH(8, 256);
    else if (n_samp <= 4096) TKA_TH(16, 256);
    else TKA_TH(32, 256);
#undef TKA_TH
    return hipGetLastError();
}
hipError_t launch_select_full(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st) {
    const dim3 grid(s.Hq, s.B);
#define TKA_SF(NT_, CPT_) hipLaunchKernelGGL((select_full_kernel<NT_, CPT_>), grid, dim3(NT_), 0, st, s, b)
    // workgroup size and register-cached scores per thread by the longest row of the call
    // (measured on batches of 256..4096 short sequences; any choice is correct)
    if (Nmax <= 512) TKA_SF(64, 8);
    else if (Nmax <= 1024) TKA_SF(64, 16);
    else if (Nmax <= 2048) TKA_SF(128, 16);
    else if (Nmax <= 4096) TKA_SF(256, 16);
    else if (Nmax <= 8192) TKA_SF(256, 32);
    else TKA_SF(kSelThreads, 8);
#undef TKA_SF
    return hipGetLastError();
}

}  // namespace tka
