// Coarse page index for the sub-linear search (the paper's methodology section leaves the kind of
// search index open; its introduction states the aim of finding the k best keys without reading all of
// them): the cache is cut into pages of 64 consecutive tokens (one tile of the key scan), and each
// page keeps a centre c (the mean of its keys, rounded to the storage type) and a radius
// r >= |k - c| for every key k of the page.  By the Cauchy-Schwarz inequality no key of the page scores more than q . c + |q| r, so a
// page whose bound stays below a head's candidate threshold cannot hold a candidate of that head,
// and the key scan skips the pages that no head of the KV group needs.  The result is exactly that
// of the plain scan.  With a bound scale beta < 1 the radius is shrunk: fewer pages are read and
// keys may be missed (approximate search).
//
//   page_ball_kernel    index build: centre, radius and |c| of the pages an append touched
//   page_filter_kernel  per decode: one bit per page and KV head (1 = scan it), 64 pages per wave
//                       scored against the group's queries with the MFMA tile routine of the scan
//   page_list_kernel    the numbers of the pages kept, ascending, and their count per key stream: the
//                       scan deals them to its waves by rank, so that every wave reads as many pages
//                       as any other whatever the pattern of the pages kept
#include "device_utils.h"
#include "internal.h"
#include "scan_tiles.h"

namespace tka {

// Rows [row0, row0 + n_rows) of the head's key stream were just written; every page they touch gets
// its ball computed from all rows it holds so far (at most 64).  One wave per page.
template <int DT>
__global__ void __launch_bounds__(256)
page_ball_kernel(const char* __restrict__ K, int D, int64_t Ncap, int64_t Pcap, int Hkv, const int32_t* __restrict__ len_dev,
                 int64_t row0_host, int64_t n_new, char* __restrict__ centres, float* __restrict__ balls) {
    constexpr int EPL = 8;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = len_dev ? (int64_t)len_dev[b] : row0_host;      // a batched append reads each sequence's length
    const int64_t n_total = row0 + n_new;
    const int64_t page = row0 / 64 + (int64_t)blockIdx.x * 4 + wave;
    if (page * 64 >= n_total) return;
    const int64_t first = page * 64;
    const int n = (int)(n_total - first < 64 ? n_total - first : 64);
    const int lpr = D / EPL, rpw = kWave / lpr;
    const int rs = lane / lpr, c = lane % lpr;
    const int64_t head = (int64_t)b * Hkv + kvh;
    const char* Kh = K + head * Ncap * D * 2;
    // mean of the page's rows
    float sum[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) sum[e] = 0.f;
    for (int r = rs; r < n; r += rpw) {
        const u32x4 raw = *reinterpret_cast<const u32x4*>(Kh + ((first + r) * D + c * EPL) * 2);
        float kf[EPL];
        Elem<DT>::widen(raw, kf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) sum[e] += kf[e];
    }
    for (int o = lpr; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sum[e] += wave_xor(sum[e], o);
    }
    // the centre as it is stored (rounded to the storage type): distances are taken from that
    float cf[EPL];
    uint32_t packed[EPL / 2];
    const float inv_n = 1.0f / (float)n;
#pragma unroll
    for (int e = 0; e < EPL; e += 2) {
        uint32_t lo, hi;
        if (DT == DT_F16) {
            const _Float16 a = (_Float16)(sum[e] * inv_n), bb = (_Float16)(sum[e + 1] * inv_n);
            cf[e] = (float)a; cf[e + 1] = (float)bb;
            lo = (uint32_t)__builtin_bit_cast(uint16_t, a); hi = (uint32_t)__builtin_bit_cast(uint16_t, bb);
        } else {
            const uint32_t ua = __float_as_uint(sum[e] * inv_n), ub = __float_as_uint(sum[e + 1] * inv_n);
            lo = (ua + 0x7FFFu + ((ua >> 16) & 1u)) >> 16;           // round to nearest even
            hi = (ub + 0x7FFFu + ((ub >> 16) & 1u)) >> 16;
            cf[e] = __uint_as_float(lo << 16); cf[e + 1] = __uint_as_float(hi << 16);
        }
        packed[e / 2] = lo | (hi << 16);
    }
    if (rs == 0) {
        u32x4 v;
        v.x = packed[0]; v.y = packed[1]; v.z = packed[2]; v.w = packed[3];
        *reinterpret_cast<u32x4*>(centres + ((head * Pcap + page) * D + c * EPL) * 2) = v;
    }
    // radius: the largest distance of a row from the stored centre; |c|
    float d2max = 0.f;
    for (int r = rs; r < n; r += rpw) {
        const u32x4 raw = *reinterpret_cast<const u32x4*>(Kh + ((first + r) * D + c * EPL) * 2);
        float kf[EPL];
        Elem<DT>::widen(raw, kf);
        float d2 = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d2 = fmaf(kf[e] - cf[e], kf[e] - cf[e], d2);
        for (int o = 1; o < lpr; o <<= 1) d2 += wave_xor(d2, o);
        d2max = fmaxf(d2max, d2);
    }
    for (int o = lpr; o < kWave; o <<= 1) d2max = fmaxf(d2max, wave_xor(d2max, o));
    float c2 = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) c2 = fmaf(cf[e], cf[e], c2);
    for (int o = 1; o < lpr; o <<= 1) c2 += wave_xor(c2, o);
    if (lane == 0) {
        // rounded up past the error of the fp32 sums (relative (D + 2) 2^-24 at most), so that the ball encloses the page
        balls[(head * Pcap + page) * 2] = sqrtf(d2max) * 1.0001f + 1e-30f;
        balls[(head * Pcap + page) * 2 + 1] = sqrtf(c2) * 1.0001f;
    }
}

// One bit per page of every (sequence, KV head): does the bound of the page reach the threshold of a head of
// the group?  A wave takes 64 pages: their centres are the "keys" of one MFMA tile.
template <int DT, int D>
__global__ void __launch_bounds__(256) page_filter_kernel(Shape sh, Bufs bf, float beta) {
    using v8 = typename Mfma<DT>::v8;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int G = sh.G, lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t head0 = (int64_t)b * sh.Hq + (int64_t)kvh * G;
    const int64_t N = prefix_len(bf.len[b], sh.window);
    const int64_t P = (N + 63) / 64;                                  // pages the search covers
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;              // 64 pages
    if (tile * 64 >= sh.page_words * 64) return;
    uint64_t* out = bf.page_mask + ((int64_t)b * sh.Hkv + kvh) * sh.page_words + tile;
    if (tile * 64 >= P) {                                             // beyond the cache: nothing to scan
        if (lane == 0) *out = 0ull;
        return;
    }
    // the centres and balls are asked for first: the query norms below wait for loads of their own
    const int64_t stream = (int64_t)b * sh.Hkv + kvh;
    const char* Ch = static_cast<const char*>(bf.page_centres) + stream * sh.page_cap * (D * 2);
    v8 cb[4][D / 32];
    tile_load<DT, D>(Ch, [&](int slot) { const int64_t p = tile * 64 + slot; return p < P ? p : P - 1; }, cb);
    const int64_t page = tile * 64 + lane;
    const float* ball = bf.page_balls + (stream * sh.page_cap + (page < P ? page : P - 1)) * 2;
    const float rad = ball[0], cn = ball[1];
    v8 qa[D / 32];
    load_query_a<DT, D>(bf.q, head0, G, qa);
    // |q| of the group's heads
    float qn[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < G; ++r) {
        float s2 = 0.f;
        for (int i = lane; i < D; i += kWave) {
            const char* qp = static_cast<const char*>(bf.q) + ((head0 + r) * D + i) * 2;
            const float v = DT == DT_F16 ? (float)*reinterpret_cast<const _Float16*>(qp)
                                         : __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(qp) << 16);
            s2 = fmaf(v, v, s2);
        }
        for (int o = 32; o > 0; o >>= 1) s2 += wave_xor(s2, o);
        qn[r] = sqrtf(s2) * 1.0001f;
    }
    const f32x4 res = tile_mac<DT, D>(cb, qa);                        // lane l: q_r . centre of page tile * 64 + l
    bool keep = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (r < G) {
            // what the scan's fp32 score of a key of the page can exceed the exact bound by, and this bound its exact value
            const float slack = 4.0f * (float)D * 5.9604645e-8f * qn[r] * (cn + rad);
            keep |= res[r] + beta * qn[r] * rad + slack >= bf.thr[head0 + r];
        }
    }
    const uint64_t m = __ballot(keep && page < P);
    if (lane == 0) *out = m;
}

// One workgroup per key stream: compacts the mask into the ascending list of the pages kept.
constexpr int kListThreads = 1024;
__global__ void __launch_bounds__(kListThreads) page_list_kernel(Shape sh, Bufs bf) {
    __shared__ uint32_t wave_tot[kListThreads / kWave];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t stream = (int64_t)blockIdx.y * sh.Hkv + blockIdx.x;
    const uint64_t* pm = bf.page_mask + stream * sh.page_words;
    int32_t* list = bf.page_list + stream * (int64_t)sh.page_words * 64;
    if (tid == 0) carry = 0u;
    __syncthreads();
    for (int w0 = 0; w0 < sh.page_words; w0 += kListThreads) {       // (uniform trip count)
        const int w = w0 + tid;
        uint64_t m = w < sh.page_words ? pm[w] : 0ull;
        const uint32_t c = (uint32_t)__popcll(m);
        uint32_t inc = c;
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t v = __shfl_up(inc, o, kWave);
            if (lane >= o) inc += v;
        }
        if (lane == kWave - 1) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t at = carry + inc - c;
        for (int i = 0; i < wave; ++i) at += wave_tot[i];
        while (m) {
            list[at++] = (int32_t)(w * 64 + __builtin_ctzll(m));
            m &= m - 1ull;
        }
        __syncthreads();
        if (tid == kListThreads - 1) carry = at;                      // the last thread's end = all pages so far
        __syncthreads();
    }
    if (tid == 0) bf.page_cnt[stream] = carry;
}

hipError_t launch_page_balls(int dtype, int D, const void* K, int64_t Ncap, int64_t Pcap, int Hkv, int B,
                             const int32_t* len_dev, int64_t row0, int64_t n_new, void* centres, float* balls, hipStream_t st) {
    if (n_new <= 0) return hipSuccess;
    const int64_t pages = (n_new + 63) / 64 + 1;                      // the first page touched may be a partly filled one
    const dim3 grid((unsigned)((pages + 3) / 4), (unsigned)Hkv, (unsigned)B);
    if (dtype == DT_F16)
        hipLaunchKernelGGL((page_ball_kernel<DT_F16>), grid, dim3(256), 0, st, static_cast<const char*>(K), D, Ncap, Pcap, Hkv,
                           len_dev, row0, n_new, static_cast<char*>(centres), balls);
    else if (dtype == DT_BF16)
        hipLaunchKernelGGL((page_ball_kernel<DT_BF16>), grid, dim3(256), 0, st, static_cast<const char*>(K), D, Ncap, Pcap, Hkv,
                           len_dev, row0, n_new, static_cast<char*>(centres), balls);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

bool pages_supported(int dtype, int D, int G) {
    return (dtype == DT_F16 || dtype == DT_BF16) && (D == 32 || D == 64 || D == 128 || D == 256) && G >= 1 && G <= 4;
}

hipError_t launch_page_filter(const Shape& s, const Bufs& b, float beta, hipStream_t st) {
    const dim3 grid((unsigned)((s.page_words + 3) / 4), (unsigned)s.Hkv, (unsigned)s.B);
#define TKA_PF(DT_, D_) hipLaunchKernelGGL((page_filter_kernel<DT_, D_>), grid, dim3(256), 0, st, s, b, beta)
    if (s.dtype == DT_F16 && s.D == 128) TKA_PF(DT_F16, 128);
    else if (s.dtype == DT_BF16 && s.D == 128) TKA_PF(DT_BF16, 128);
    else if (s.dtype == DT_F16 && s.D == 64) TKA_PF(DT_F16, 64);
    else if (s.dtype == DT_BF16 && s.D == 64) TKA_PF(DT_BF16, 64);
    else if (s.dtype == DT_F16 && s.D == 256) TKA_PF(DT_F16, 256);
    else if (s.dtype == DT_BF16 && s.D == 256) TKA_PF(DT_BF16, 256);
    else if (s.dtype == DT_F16 && s.D == 32) TKA_PF(DT_F16, 32);
    else if (s.dtype == DT_BF16 && s.D == 32) TKA_PF(DT_BF16, 32);
    else return hipErrorInvalidValue;
#undef TKA_PF
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(page_list_kernel, dim3((unsigned)s.Hkv, (unsigned)s.B), dim3(kListThreads), 0, st, s, b);
    return hipGetLastError();
}

}  // namespace tka
