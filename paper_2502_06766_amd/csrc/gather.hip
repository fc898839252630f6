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
#include "internal.h"

namespace tka {

struct GatherShared {
    float red[4][256 + 1];
    float sc[kGatherRows];     // window chunk: raw scores of its rows
    float q[256];              // window chunk: the query row in fp32
    float wmax[4];
};

// Weighted sum of value rows j in [j0, j1): row(j) gives the cache position, weight(j) its
// softmax numerator.  Leaves the partial of this workgroup in slot `slot` of the head.
// With `direct` (the head has this one partial only) the normalised result goes straight to
// `out` / `lse` and no merge kernel follows.
template <int DT, class RowFn, class WeightFn>
__device__ __forceinline__ void wg_weighted_rows(const Shape& sh, const Bufs& bf, int64_t bh, const char* Vh, int j0,
                                                 int j1, RowFn row, WeightFn weight, float m_ref, int slot,
                                                 GatherShared& sm, bool direct = false, float scale = 0.f) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    const int D = sh.D;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int lpr = D / EPL;                 // lanes per value row
    const int rpw = kWave / lpr;             // rows per wave per load
    const int rs = lane / lpr, c = lane % lpr;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float lsum = 0.f;
    // U independent rows per lane group at a time (a row's position, its weight,
    // then the row itself are dependent loads: one at a time is latency-bound for small k)
    constexpr int U = 4;
    const int step = 4 * rpw;
    for (int j = j0 + wave * rpw + rs; j < j1; j += U * step) {
        int64_t r[U];
        float w[U];
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = j + u * step;
            const bool ok = jj < j1;
            r[u] = row(ok ? jj : j);
            w[u] = ok ? weight(jj) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            raw[u] = *reinterpret_cast<const u32x4*>(Vh + (r[u] * D + c * EPL) * Elem<DT>::kBytes);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[EPL];
            Elem<DT>::widen(raw[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(w[u], vf[e], acc[e]);
            lsum += w[u];
        }
    }
    // add the row slots of the wave together
    for (int o = lpr; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += wave_xor(acc[e], o);
        lsum += wave_xor(lsum, o);
    }
    if (rs == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm.red[wave][c * EPL + e] = acc[e];
        if (c == 0) sm.red[wave][256] = lsum;
    }
    __syncthreads();
    if (direct) {
        const float l = (sm.red[0][256] + sm.red[1][256]) + (sm.red[2][256] + sm.red[3][256]);
        for (int t = threadIdx.x; t < D; t += blockDim.x)
            bf.out[bh * D + t] = ((sm.red[0][t] + sm.red[1][t]) + (sm.red[2][t] + sm.red[3][t])) / l;
        if (threadIdx.x == 0 && bf.lse) bf.lse[bh] = m_ref * scale + logf(l);
        return;
    }
    float* pa = bf.part_acc + (bh * sh.n_chunk_cap + slot) * D;
    for (int t = threadIdx.x; t < D; t += blockDim.x)
        pa[t] = (sm.red[0][t] + sm.red[1][t]) + (sm.red[2][t] + sm.red[3][t]);
    if (threadIdx.x == 0) {
        bf.part_l[bh * sh.n_chunk_cap + slot] =
            (sm.red[0][256] + sm.red[1][256]) + (sm.red[2][256] + sm.red[3][256]);
        bf.part_m[bh * sh.n_chunk_cap + slot] = m_ref;
    }
}

__device__ __forceinline__ void mark_empty(const Shape& sh, const Bufs& bf, int64_t bh, int slot) {
    if (threadIdx.x == 0) {
        bf.part_l[bh * sh.n_chunk_cap + slot] = 0.f;
        bf.part_m[bh * sh.n_chunk_cap + slot] = -INFINITY;
    }
}

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

// slots [slot0, slot0 + ceil(window / kGatherRows)): the always-attended recent tokens,
// scored here with plain FMAs (a few thousand rows at most)
template <int DT>
__global__ void __launch_bounds__(256) window_partial_kernel(Shape sh, Bufs bf, float scale_log2e, int slot0) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    __shared__ GatherShared sm;
    const int chunk_id = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int64_t N = visible_len(sh, bf, b);
    const int64_t P = prefix_len(N, sh.window);
    const int W = (int)(N - P);
    const int j0 = chunk_id * kGatherRows;
    if (j0 >= W) { mark_empty(sh, bf, bh, slot0 + chunk_id); return; }
    const int j1 = j0 + kGatherRows < W ? j0 + kGatherRows : W;
    const int64_t head_off = ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * D * Elem<DT>::kBytes;
    const char* Kh = static_cast<const char*>(bf.K) + head_off;
    const char* Vh = static_cast<const char*>(bf.V) + head_off;

    for (int i = threadIdx.x; i < D; i += blockDim.x) {
        const char* qp = static_cast<const char*>(bf.q) + (bh * D + i) * Elem<DT>::kBytes;
        float v;
        if (DT == DT_F32) v = *reinterpret_cast<const float*>(qp);
        else if (DT == DT_F16) v = (float)*reinterpret_cast<const _Float16*>(qp);
        else v = __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(qp) << 16);
        sm.q[i] = v;
    }
    __syncthreads();
    // scores of the chunk's rows and their maximum
    const int lpr = D / EPL, rows_per_pass = 256 / lpr;
    const int rs = threadIdx.x / lpr, c = threadIdx.x % lpr;
    float mx = -INFINITY;
    for (int j = j0; j < j1; j += rows_per_pass) {
        const int jj = j + rs;
        const bool valid = jj < j1;
        const int64_t r = P + (valid ? jj : j1 - 1);
        const u32x4 raw = *reinterpret_cast<const u32x4*>(Kh + (r * D + c * EPL) * Elem<DT>::kBytes);
        float kf[EPL];
        Elem<DT>::widen(raw, kf);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc = fmaf(kf[e], sm.q[c * EPL + e], acc);
        for (int o = 1; o < lpr; o <<= 1) acc += wave_xor(acc, o);
        if (valid) {
            if (c == 0) sm.sc[jj - j0] = acc;
            mx = fmaxf(mx, acc);
        }
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, wave_xor(mx, o));
    if (lane_id() == 0) sm.wmax[threadIdx.x >> 6] = mx;
    __syncthreads();
    const float m = fmaxf(fmaxf(sm.wmax[0], sm.wmax[1]), fmaxf(sm.wmax[2], sm.wmax[3]));
    wg_weighted_rows<DT>(sh, bf, bh, Vh, j0, j1, [&](int j) { return P + j; },
                         [&](int j) { return exp2f((sm.sc[j - j0] - m) * scale_log2e); }, m, slot0 + chunk_id, sm);
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
hipError_t launch_window_partials(const Shape& s, const Bufs& b, int slot0, hipStream_t st) {
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
