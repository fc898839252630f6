// Attention over the selected rows: out = Softmax(vals / sqrt(d)) . V[I]
// (the attention step of Algorithm 1 of arXiv 2502.06766, with the 1/sqrt(d) scale of
// Eq. 1), max-subtracted, fp32 accumulate.  The k rows of a head are split over
// workgroups of kGatherRows rows; each produces an unnormalised partial sum, its weight
// total and the score the weights are relative to (the head's largest selected score,
// known from the selection).  Optionally the most recent `window` tokens (Algorithm 1's
// K_gen / V_gen, attended densely) add further partials, each relative to its own chunk
// maximum.  A last small kernel merges all partials of a head in a fixed order with the
// usual log-sum-exp rescaling and normalises: one softmax over retrieved + window scores.
#include "device_utils.h"
#include "gather_common.h"
#include "internal.h"

namespace tka {

// slots [0, ceil(k / kGatherRows)): the retrieved rows
template <int DT>
__global__ void __launch_bounds__(256) gather_partial_kernel(Shape sh, Bufs bf, float scale_log2e, float scale,
                                                             int direct) {
    __shared__ GatherShared sm;
    const int chunk_id = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int64_t P = prefix_len(visible_len(sh, bf, b), sh.window);
    const int k_eff = sh.k < P ? sh.k : (int)P;
    const int j0 = chunk_id * kGatherRows;
    if (j0 >= k_eff) { mark_empty(sh, bf, bh, chunk_id); return; }
    const int j1 = j0 + kGatherRows < k_eff ? j0 + kGatherRows : k_eff;
    const char* Vh = static_cast<const char*>(bf.V) +
                     ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * sh.D * Elem<DT>::kBytes;
    const int32_t* idx = bf.sel_idx + bh * sh.k;
    const float* val = bf.sel_val + bh * sh.k;
    const float m = bf.hmax[bh];
    wg_weighted_rows<DT>(sh, bf, bh, Vh, j0, j1, [&](int j) { return (int64_t)idx[j]; },
                         [&](int j) { return exp2f((val[j] - m) * scale_log2e); }, m, chunk_id, sm, direct != 0, scale);
}

// slots [slot0, slot0 + ceil(window / kGatherRows)): the always-attended recent tokens
template <int DT>
__global__ void __launch_bounds__(256) window_partial_kernel(Shape sh, Bufs bf, float scale_log2e, int slot0) {
    __shared__ GatherShared sm;
    window_chunk<DT>(sh, bf, scale_log2e, blockIdx.x, blockIdx.y, blockIdx.z, slot0 + blockIdx.x, sm);
}

constexpr int kCombineSlots = 1024;   // partial slots whose rescale factors are staged in LDS

// Without a window every partial of a head is relative to the same score (the head's
// largest selected one): plain sums, one round of loads.
__global__ void __launch_bounds__(256) gather_sum_kernel(Shape sh, Bufs bf, float scale) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t N = visible_len(sh, bf, b);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const int nch = (k_eff + kGatherRows - 1) / kGatherRows;
    __shared__ float red[256];
    __shared__ float wred[4];
    const int parts = 256 / D, e = tid % D, part = tid / D;
    const float* pa = bf.part_acc + bh * sh.n_chunk_cap * (int64_t)D + e;
    float a = 0.f;
#pragma unroll 8
    for (int ch = part; ch < nch; ch += parts) a += pa[(int64_t)ch * D];
    float l = 0.f;
    for (int ch = tid; ch < nch; ch += 256) l += bf.part_l[bh * sh.n_chunk_cap + ch];
    for (int o = 32; o > 0; o >>= 1) l += wave_xor(l, o);      // fixed tree: same result every run
    if (lane == 0) wred[wave] = l;
    red[tid] = a;
    __syncthreads();
    if (tid < D) {
        const float lt = (wred[0] + wred[1]) + (wred[2] + wred[3]);
        float at = 0.f;
        for (int p = 0; p < parts; ++p) at += red[p * D + e];
        bf.out[bh * D + e] = at / lt;
        if (tid == 0 && bf.lse) bf.lse[bh] = bf.hmax[bh] * scale + logf(lt);
    }
}

// With a window the partials carry their own reference scores: log-sum-exp merge.
__global__ void __launch_bounds__(256) gather_combine_kernel(Shape sh, Bufs bf, float scale, float scale_log2e,
                                                             int n_slots) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    __shared__ float red[256];
    __shared__ float fac[kCombineSlots];
    __shared__ float wred[4];
    const float* pl = bf.part_l + bh * sh.n_chunk_cap;
    const float* pm = bf.part_m + bh * sh.n_chunk_cap;
    // reference score of the merged softmax: the largest one any non-empty partial used
    float M = -INFINITY;
    for (int s = tid; s < n_slots; s += 256)
        if (pl[s] > 0.f) M = fmaxf(M, pm[s]);
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, wave_xor(M, o));
    if (lane == 0) wred[wave] = M;
    __syncthreads();
    M = fmaxf(fmaxf(wred[0], wred[1]), fmaxf(wred[2], wred[3]));
    __syncthreads();
    // per-slot rescale factor 2^((m_s - M) scale log2e) (0 for an empty slot) and the weight total
    float l = 0.f;
    for (int s = tid; s < n_slots; s += 256) {
        const float ls = pl[s];
        const float f = ls > 0.f ? exp2f((pm[s] - M) * scale_log2e) : 0.f;
        if (s < kCombineSlots) fac[s] = f;
        l = fmaf(ls, f, l);
    }
    for (int o = 32; o > 0; o >>= 1) l += wave_xor(l, o);      // fixed tree: same result every run
    if (lane == 0) wred[wave] = l;
    __syncthreads();
    const float lt = (wred[0] + wred[1]) + (wred[2] + wred[3]);
    // 256 / D threads share an output element, each adds every (256 / D)-th partial
    const int parts = 256 / D, e = tid % D, part = tid / D;
    const float* pa = bf.part_acc + bh * sh.n_chunk_cap * (int64_t)D + e;
    float a = 0.f;
#pragma unroll 8
    for (int s = part; s < n_slots; s += parts) {
        const float f = s < kCombineSlots ? fac[s] : (pl[s] > 0.f ? exp2f((pm[s] - M) * scale_log2e) : 0.f);
        if (f > 0.f) a = fmaf(pa[(int64_t)s * D], f, a);
    }
    red[tid] = a;
    __syncthreads();
    if (tid < D) {
        float at = 0.f;
        for (int p = 0; p < parts; ++p) at += red[p * D + e];
        bf.out[bh * D + e] = at / lt;
        if (tid == 0 && bf.lse) bf.lse[bh] = M * scale + logf(lt);
    }
}

// Partial sums over the recent-token window of every head into the slots slot0, slot0 + 1, ... (one per
// kGatherRows tokens), each relative to its own largest score.
static hipError_t launch_window_partials(const Shape& s, const Bufs& b, int slot0, hipStream_t st) {
    const float scale_log2e = (1.0f / sqrtf((float)s.D)) * 1.4426950408889634f;
    const int nwin = (s.window + kGatherRows - 1) / kGatherRows;
    if (nwin == 0) return hipSuccess;
    dim3 wgrid((unsigned)nwin, (unsigned)s.Hq, (unsigned)s.B);
    if (s.dtype == DT_F32)
        hipLaunchKernelGGL((window_partial_kernel<DT_F32>), wgrid, dim3(256), 0, st, s, b, scale_log2e, slot0);
    else if (s.dtype == DT_F16)
        hipLaunchKernelGGL((window_partial_kernel<DT_F16>), wgrid, dim3(256), 0, st, s, b, scale_log2e, slot0);
    else
        hipLaunchKernelGGL((window_partial_kernel<DT_BF16>), wgrid, dim3(256), 0, st, s, b, scale_log2e, slot0);
    return hipGetLastError();
}

hipError_t launch_gather(const Shape& s, const Bufs& b, hipStream_t st) {
    const float scale = 1.0f / sqrtf((float)s.D);
    const float scale_log2e = scale * 1.4426950408889634f;
    const int nch = (s.k + kGatherRows - 1) / kGatherRows;
    const int nwin = (s.window + kGatherRows - 1) / kGatherRows;
    dim3 grid((unsigned)nch, (unsigned)s.Hq, (unsigned)s.B);
    // one chunk per head and no window: the gather writes the result itself (k_eff >= 1 for every sequence)
    const int direct = nch == 1 && nwin == 0 ? 1 : 0;
    if (s.dtype == DT_F32)
        hipLaunchKernelGGL((gather_partial_kernel<DT_F32>), grid, dim3(256), 0, st, s, b, scale_log2e, scale, direct);
    else if (s.dtype == DT_F16)
        hipLaunchKernelGGL((gather_partial_kernel<DT_F16>), grid, dim3(256), 0, st, s, b, scale_log2e, scale, direct);
    else
        hipLaunchKernelGGL((gather_partial_kernel<DT_BF16>), grid, dim3(256), 0, st, s, b, scale_log2e, scale, direct);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (nwin > 0) {
        e = launch_window_partials(s, b, nch, st);
        if (e != hipSuccess) return e;
    }
    if (nwin > 0)
        hipLaunchKernelGGL(gather_combine_kernel, dim3(s.Hq, s.B), dim3(256), 0, st, s, b, scale, scale_log2e,
                           nch + nwin);
    else if (!direct)
        hipLaunchKernelGGL(gather_sum_kernel, dim3(s.Hq, s.B), dim3(256), 0, st, s, b, scale);
    return hipGetLastError();
}

}  // namespace tka
