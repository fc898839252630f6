// Attention over the selected rows: out = Softmax(vals / sqrt(d)) . V[I]
// (the attention step of Algorithm 1 of arXiv 2502.06766, with the 1/sqrt(d) scale of
// Eq. 1), max-subtracted, fp32 accumulate.  The k rows of a head are split over
// workgroups of kGatherRows rows; each produces an unnormalised partial sum and weight
// total relative to the head's largest score (known from the selection), and a second
// small kernel adds the partials in a fixed order and normalises.
#include "device_utils.h"
#include "internal.h"

namespace tka {

template <int DT>
__global__ void __launch_bounds__(256) gather_partial_kernel(Shape sh, Bufs bf, float scale_log2e) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    const int chunk_id = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const int j0 = chunk_id * kGatherRows;
    if (j0 >= k_eff) return;
    const int j1 = j0 + kGatherRows < k_eff ? j0 + kGatherRows : k_eff;

    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int lpr = D / EPL;                 // lanes per value row
    const int rpw = kWave / lpr;             // rows per wave per load
    const int slot = lane / lpr, c = lane % lpr;
    const int kvh = h / sh.G;
    const char* Vh = static_cast<const char*>(bf.V) +
                     ((int64_t)b * sh.Hkv + kvh) * sh.Ncap * D * Elem<DT>::kBytes;
    const int32_t* idx = bf.sel_idx + bh * sh.k;
    const float* val = bf.sel_val + bh * sh.k;
    const float m = bf.hmax[bh];

    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float lsum = 0.f;
    for (int j = j0 + wave * rpw + slot; j < j1; j += 4 * rpw) {
        const int64_t row = idx[j];
        const float w = exp2f((val[j] - m) * scale_log2e);
        const u32x4 raw = *reinterpret_cast<const u32x4*>(Vh + (row * D + c * EPL) * Elem<DT>::kBytes);
        float vf[EPL];
        Elem<DT>::widen(raw, vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(w, vf[e], acc[e]);
        lsum += w;
    }
    // add the row slots of the wave together
    for (int o = lpr; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += wave_xor(acc[e], o);
        lsum += wave_xor(lsum, o);
    }
    __shared__ float red[4][256 + 1];
    if (slot == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) red[wave][c * EPL + e] = acc[e];
        if (c == 0) red[wave][256] = lsum;
    }
    __syncthreads();
    float* pa = bf.part_acc + (bh * sh.n_chunk_cap + chunk_id) * D;
    for (int t = threadIdx.x; t < D; t += blockDim.x)
        pa[t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    if (threadIdx.x == 0)
        bf.part_l[bh * sh.n_chunk_cap + chunk_id] = (red[0][256] + red[1][256]) + (red[2][256] + red[3][256]);
}

__global__ void __launch_bounds__(256) gather_combine_kernel(Shape sh, Bufs bf, float scale) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int64_t N = bf.len[b];
    const int k_eff = sh.k < N ? sh.k : (int)N;
    const int nch = (k_eff + kGatherRows - 1) / kGatherRows;
    // 256 / D threads share an output element, each adds every (256 / D)-th partial
    const int parts = 256 / D, e = threadIdx.x % D, part = threadIdx.x / D;
    __shared__ float red[256];
    __shared__ float lred[256];
    const float* pa = bf.part_acc + bh * sh.n_chunk_cap * (int64_t)D + e;
    float a = 0.f;
#pragma unroll 8
    for (int ch = part; ch < nch; ch += parts) a += pa[(int64_t)ch * D];
    float l = 0.f;
    for (int ch = threadIdx.x; ch < nch; ch += 256) l += bf.part_l[bh * sh.n_chunk_cap + ch];
    red[threadIdx.x] = a;
    lred[threadIdx.x] = l;
    __syncthreads();
    if (threadIdx.x < D) {
        float lt = 0.f;
        for (int i = 0; i < 256; ++i) lt += lred[i];      // fixed order
        float at = 0.f;
        for (int p = 0; p < parts; ++p) at += red[p * D + e];
        bf.out[bh * D + e] = at / lt;
        if (threadIdx.x == 0 && bf.lse) bf.lse[bh] = bf.hmax[bh] * scale + logf(lt);
    }
}

hipError_t launch_gather(const Shape& s, const Bufs& b, hipStream_t st) {
    const float scale = 1.0f / sqrtf((float)s.D);
    const float scale_log2e = scale * 1.4426950408889634f;
    const int nch = (s.k + kGatherRows - 1) / kGatherRows;
    dim3 grid((unsigned)nch, (unsigned)s.Hq, (unsigned)s.B);
    if (s.dtype == DT_F32)
        hipLaunchKernelGGL((gather_partial_kernel<DT_F32>), grid, dim3(256), 0, st, s, b, scale_log2e);
    else if (s.dtype == DT_F16)
        hipLaunchKernelGGL((gather_partial_kernel<DT_F16>), grid, dim3(256), 0, st, s, b, scale_log2e);
    else
        hipLaunchKernelGGL((gather_partial_kernel<DT_BF16>), grid, dim3(256), 0, st, s, b, scale_log2e);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gather_combine_kernel, dim3(s.Hq, s.B), dim3(256), 0, st, s, b, scale);
    return hipGetLastError();
}

}  // namespace tka
