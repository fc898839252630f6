// Pieces of the weighted value sum shared by the gather kernels and the tail of the filtered path:
// the workgroup-wide weighted sum of value rows (one partial of a head's softmax-weighted sum), and the
// partial of one chunk of the always-attended recent tokens (Algorithm 1's K_gen / V_gen of
// arXiv 2502.06766, attended densely).  Workgroups of 256 threads.
#pragma once
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

// Partial `slot` of head (b, h): chunk `chunk_id` (kGatherRows tokens) of the recent-token window of the
// head's sequence, scored here with plain FMAs (a few thousand rows at most), weights relative to the
// chunk's own largest score.  An empty partial if the sequence's window does not reach the chunk.
template <int DT>
__device__ __forceinline__ void window_chunk(const Shape& sh, const Bufs& bf, float scale_log2e, int chunk_id, int h, int b,
                                             int slot, GatherShared& sm) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int64_t N = visible_len(sh, bf, b);
    const int64_t P = prefix_len(N, sh.window);
    const int W = (int)(N - P);
    const int j0 = chunk_id * kGatherRows;
    if (j0 >= W) { mark_empty(sh, bf, bh, slot); return; }
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
    float qf[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = sm.q[c * EPL + e];
    constexpr int UW = 4;          // key rows in flight per lane (one at a time is a chain of trips to memory)
    for (int j = j0; j < j1; j += UW * rows_per_pass) {
        u32x4 raw[UW];
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int jj = j + u * rows_per_pass + rs;
            const int64_t r = P + (jj < j1 ? jj : j1 - 1);
            raw[u] = *reinterpret_cast<const u32x4*>(Kh + (r * D + c * EPL) * Elem<DT>::kBytes);
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int jj = j + u * rows_per_pass + rs;
            float kf[EPL];
            Elem<DT>::widen(raw[u], kf);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc = fmaf(kf[e], qf[e], acc);
            for (int o = 1; o < lpr; o <<= 1) acc += wave_xor(acc, o);
            if (jj < j1) {
                if (c == 0) sm.sc[jj - j0] = acc;
                mx = fmaxf(mx, acc);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, wave_xor(mx, o));
    if (lane_id() == 0) sm.wmax[threadIdx.x >> 6] = mx;
    __syncthreads();
    const float m = fmaxf(fmaxf(sm.wmax[0], sm.wmax[1]), fmaxf(sm.wmax[2], sm.wmax[3]));
    wg_weighted_rows<DT>(sh, bf, bh, Vh, j0, j1, [&](int j) { return P + j; },
                         [&](int j) { return exp2f((sm.sc[j - j0] - m) * scale_log2e); }, m, slot, sm);
}

}  // namespace tka
