// Compressed key index: every key row is kept a second time as int8 codes with one fp32
// scale per row (the search index of the paper's methodology section need not be the plain
// key list; this is the compressed-list kind: approximate search, exact refinement).
//
//   code_c = rint(x_c * (127 / amax)),  scale = amax / 127,  amax = max_c |x_c|
//   (rows with amax < 2^-100 are coded as all zeros with scale 0)
//   s~ = float(sum_c codeq_c * codeK_c) * (scale_q * scale_K)
//
// The scan over the codes is the grouped MFMA scan again with v_mfma_i32_16x16x64_i8 and
// half the bytes per key; the candidates it keeps carry approximate scores, which
// rerank_kernel replaces by exact fp32 dot products with the 16-bit rows before the exact
// selection runs.  A key whose approximate score falls below the (lowered) threshold
// although its exact score belongs to the top k is lost: the result is approximate, with
// recall measured against the exact path.
#include "device_utils.h"
#include "internal.h"
#include "scan_common.h"

namespace tka {

typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr float kTinyRow = 7.888609052210118e-31f;   // 2^-100

// ---------------------------------------------------------------------------------------
// Row coding.  A row of D elements is spread over D / 8 lanes (16-bit storage, 16 bytes
// per lane); row r is row r % rows_per_head of head r / rows_per_head.
// ---------------------------------------------------------------------------------------
template <int DT>
__global__ void __launch_bounds__(256)
quantize_rows_kernel(const char* __restrict__ src, int64_t rows_per_head, int64_t src_head_stride_bytes,
                     int64_t n_rows, int D, int8_t* __restrict__ dst, float* __restrict__ scale,
                     int64_t dst_head_stride_rows) {
    constexpr int EPL = Elem<DT>::kPerLoad;          // 8 for 16-bit storage
    const int lpr = D / EPL;                         // lanes per row: 8, 16 or 32
    const int rows_per_pass = 256 / lpr;
    const int rs = threadIdx.x / lpr, c = threadIdx.x % lpr;
    for (int64_t base = (int64_t)blockIdx.x * rows_per_pass; base < n_rows; base += (int64_t)gridDim.x * rows_per_pass) {
        const int64_t r = base + rs;
        const bool valid = r < n_rows;
        const int64_t rr = valid ? r : n_rows - 1;
        const int64_t head = rr / rows_per_head, t = rr - head * rows_per_head;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(src + head * src_head_stride_bytes +
                                                          (t * D + c * EPL) * Elem<DT>::kBytes);
        float x[EPL];
        Elem<DT>::widen(raw, x);
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(x[e]));
        for (int o = 1; o < lpr; o <<= 1) amax = fmaxf(amax, wave_xor(amax, o));
        const bool live = amax >= kTinyRow;
        const float inv = live ? 127.0f / amax : 0.f;
        uint32_t w[EPL / 4];
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            uint32_t p = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int code = (int)rintf(x[4 * i + e] * inv);
                p |= ((uint32_t)code & 0xFFu) << (8 * e);
            }
            w[i] = p;
        }
        if (valid) {
            const int64_t drow = head * dst_head_stride_rows + t;
            uint32_t* d = reinterpret_cast<uint32_t*>(dst + drow * D + c * EPL);
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) d[i] = w[i];
            if (c == 0) scale[drow] = live ? amax / 127.0f : 0.f;
        }
    }
}

// Row coding of the tokens a batched append adds: source rows [B][n_new][Hkv] (contiguous),
// row (b, t, h) is coded into row len[b] + t of (b, h) of the layer's index.
template <int DT>
__global__ void __launch_bounds__(256)
quantize_step_kernel(const char* __restrict__ src, int64_t n_rows, int64_t n_new, int Hkv, int64_t Ncap, int D,
                     const int32_t* __restrict__ len, int8_t* __restrict__ dst, float* __restrict__ scale) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    const int lpr = D / EPL;
    const int rows_per_pass = 256 / lpr;
    const int rs = threadIdx.x / lpr, c = threadIdx.x % lpr;
    for (int64_t base = (int64_t)blockIdx.x * rows_per_pass; base < n_rows; base += (int64_t)gridDim.x * rows_per_pass) {
        const int64_t r = base + rs;
        const bool valid = r < n_rows;
        const int64_t rr = valid ? r : n_rows - 1;
        const int h = (int)(rr % Hkv);
        const int64_t bt = rr / Hkv, t = bt % n_new, b = bt / n_new;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(src + (rr * D + c * EPL) * Elem<DT>::kBytes);
        float x[EPL];
        Elem<DT>::widen(raw, x);
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(x[e]));
        for (int o = 1; o < lpr; o <<= 1) amax = fmaxf(amax, wave_xor(amax, o));
        const bool live = amax >= kTinyRow;
        const float inv = live ? 127.0f / amax : 0.f;
        uint32_t w[EPL / 4];
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            uint32_t p = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int code = (int)rintf(x[4 * i + e] * inv);
                p |= ((uint32_t)code & 0xFFu) << (8 * e);
            }
            w[i] = p;
        }
        if (valid) {
            const int64_t drow = (b * Hkv + h) * Ncap + (int64_t)len[b] + t;
            uint32_t* d = reinterpret_cast<uint32_t*>(dst + drow * D + c * EPL);
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) d[i] = w[i];
            if (c == 0) scale[drow] = live ? amax / 127.0f : 0.f;
        }
    }
}

hipError_t launch_quantize_step(int dtype, int D, const void* src, int B, int64_t n_new, int Hkv, int64_t Ncap,
                                const int32_t* len, int8_t* codes, float* scale, hipStream_t st) {
    const int64_t n_rows = (int64_t)B * n_new * Hkv;
    if (n_rows <= 0) return hipSuccess;
    const int rows_per_pass = 256 / (D / 8);
    int64_t blocks = (n_rows + rows_per_pass - 1) / rows_per_pass;
    if (blocks > 65536) blocks = 65536;
    if (dtype == DT_F16)
        hipLaunchKernelGGL((quantize_step_kernel<DT_F16>), dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const char*>(src), n_rows, n_new, Hkv, Ncap, D, len, codes, scale);
    else if (dtype == DT_BF16)
        hipLaunchKernelGGL((quantize_step_kernel<DT_BF16>), dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const char*>(src), n_rows, n_new, Hkv, Ncap, D, len, codes, scale);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// A small batched append on a cache with the int8 index in one launch: one workgroup places the new key and
// value rows, codes the key rows, and bumps the lengths once all its threads have used them.
constexpr int kAppendSmall8Threads = 1024;
template <int DT>
__global__ void __launch_bounds__(kAppendSmall8Threads)
append_step_small8_kernel(const char* __restrict__ ksrc, const char* __restrict__ vsrc, char* __restrict__ kdst,
                          char* __restrict__ vdst, int64_t head_b, int64_t n_rows, int64_t n_new, int Hkv, int64_t Ncap,
                          int D, int B, int32_t* len, int8_t* __restrict__ dst, float* __restrict__ scale) {
    constexpr int EPL = Elem<DT>::kPerLoad;          // 8: the index codes 16-bit caches
    const int lpr = D / EPL;
    const int rows_per_pass = kAppendSmall8Threads / lpr;
    const int rs = threadIdx.x / lpr, c = threadIdx.x % lpr;
    for (int64_t base = 0; base < n_rows; base += rows_per_pass) {
        const int64_t r = base + rs;
        const bool valid = r < n_rows;
        const int64_t rr = valid ? r : n_rows - 1;
        const int h = (int)(rr % Hkv);
        const int64_t bt = rr / Hkv, t = bt % n_new, b = bt / n_new;
        const int64_t s_o = (rr * D + c * EPL) * Elem<DT>::kBytes;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(ksrc + s_o);
        const u32x4 rawv = *reinterpret_cast<const u32x4*>(vsrc + s_o);
        const int64_t row = (int64_t)len[b] + t;
        float x[EPL];
        Elem<DT>::widen(raw, x);
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(x[e]));
        for (int o = 1; o < lpr; o <<= 1) amax = fmaxf(amax, wave_xor(amax, o));
        const bool live = amax >= kTinyRow;
        const float inv = live ? 127.0f / amax : 0.f;
        uint32_t w[EPL / 4];
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            uint32_t p = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int code = (int)rintf(x[4 * i + e] * inv);
                p |= ((uint32_t)code & 0xFFu) << (8 * e);
            }
            w[i] = p;
        }
        if (valid) {
            const int64_t d_o = (b * Hkv + h) * head_b + (row * D + c * EPL) * Elem<DT>::kBytes;
            *reinterpret_cast<u32x4*>(kdst + d_o) = raw;
            *reinterpret_cast<u32x4*>(vdst + d_o) = rawv;
            const int64_t drow = (b * Hkv + h) * Ncap + row;
            uint32_t* d = reinterpret_cast<uint32_t*>(dst + drow * D + c * EPL);
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) d[i] = w[i];
            if (c == 0) scale[drow] = live ? amax / 127.0f : 0.f;
        }
    }
    __syncthreads();            // every thread has used the lengths it needed
    for (int b = threadIdx.x; b < B; b += kAppendSmall8Threads) len[b] += (int32_t)n_new;
}

hipError_t launch_append_step_small8(int dtype, int D, const void* ksrc, const void* vsrc, void* kdst, void* vdst,
                                     int64_t head_bytes, int B, int64_t n_new, int Hkv, int64_t Ncap, int32_t* len,
                                     int8_t* codes, float* scale, hipStream_t st) {
    const int64_t n_rows = (int64_t)B * n_new * Hkv;
#define TKA_AS8(DT_)                                                                                                     \
    hipLaunchKernelGGL((append_step_small8_kernel<DT_>), dim3(1), dim3(kAppendSmall8Threads), 0, st,                    \
                       static_cast<const char*>(ksrc), static_cast<const char*>(vsrc), static_cast<char*>(kdst),        \
                       static_cast<char*>(vdst), head_bytes, n_rows, n_new, Hkv, Ncap, D, B, len, codes, scale)
    if (dtype == DT_F16) TKA_AS8(DT_F16);
    else if (dtype == DT_BF16) TKA_AS8(DT_BF16);
    else return hipErrorInvalidValue;
#undef TKA_AS8
    return hipGetLastError();
}

bool index8_supported(int dtype, int D, int G) {
    return (dtype == DT_F16 || dtype == DT_BF16) && (D == 64 || D == 128 || D == 256) && G >= 1 && G <= 4;
}

hipError_t launch_quantize_rows(int dtype, int D, const void* src, int64_t rows_per_head, int64_t src_head_stride_bytes,
                                int n_heads, int8_t* dst, float* scale, int64_t dst_head_stride_rows, hipStream_t st) {
    const int64_t n_rows = rows_per_head * n_heads;
    if (n_rows <= 0) return hipSuccess;
    const int rows_per_pass = 256 / (D / 8);
    int64_t blocks = (n_rows + rows_per_pass - 1) / rows_per_pass;
    if (blocks > 65536) blocks = 65536;
    if (dtype == DT_F16)
        hipLaunchKernelGGL((quantize_rows_kernel<DT_F16>), dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const char*>(src), rows_per_head, src_head_stride_bytes, n_rows, D, dst, scale,
                           dst_head_stride_rows);
    else if (dtype == DT_BF16)
        hipLaunchKernelGGL((quantize_rows_kernel<DT_BF16>), dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const char*>(src), rows_per_head, src_head_stride_bytes, n_rows, D, dst, scale,
                           dst_head_stride_rows);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Scan over the codes (grouped layout: one query, up to four heads per KV head).
// ---------------------------------------------------------------------------------------
// Codes of a 64-key tile in operand-B layout (lane (j, n) holds the 16-byte chunk 4 s + j of
// key 16 g + n) and the scale of key `lane`.
template <int D, class RowFn>
__device__ __forceinline__ void tile_load8(const int8_t* Kh, const float* Sh, RowFn rowfn, i32x4 (&b)[4][D / 64],
                                           float& ks) {
    constexpr int KS = D / 64;
    const int lane = lane_id();
    const int j = lane >> 4, n = lane & 15;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t row = rowfn(16 * g + n);
        const i32x4* p = reinterpret_cast<const i32x4*>(Kh + row * D) + j;
#pragma unroll
        for (int s = 0; s < KS; ++s) b[g][s] = p[4 * s];
    }
    ks = Sh[rowfn(lane)];
}

// Integer dot products of the tile: lane l gets res[r] = codes(q_{head0 + r}) . codes(K[row(l)]).
template <int D>
__device__ __forceinline__ i32x4 tile_mac8(const i32x4 (&b)[4][D / 64], const i32x4 (&qa)[D / 64]) {
    constexpr int KS = D / 64;
    const int j = lane_id() >> 4;
    i32x4 c[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        c[g] = i32x4{0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) c[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa[s], b[g][s], c[g], 0, 0, 0);
    }
    i32x4 res;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int lo = (j & 1) ? c[1][r] : c[0][r];
        const int hi = (j & 1) ? c[3][r] : c[2][r];
        res[r] = (j & 2) ? hi : lo;
    }
    return res;
}

template <int D, int MODE>
__global__ void __launch_bounds__(kScanWaves* kWave)
scan8_kernel(Shape sh, Bufs bf, int tiles_per_wave, float* dst) {
    constexpr int KS = D / 64;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int G = sh.G;
    const int64_t head0 = (int64_t)b * sh.Hq + (int64_t)kvh * G;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t N = prefix_len(bf.len[b], sh.window);

    int64_t n_items = N;
    int stride = 1;
    if (MODE == MODE_SAMPLE) {
        if (N == 0) return;
        Plan pl = make_plan(N, sh.k < N ? sh.k : (int)N, 1);
        n_items = pl.n_samp;
        stride = pl.stride;
    }
    const int64_t n_tiles_all = (n_items + 63) / 64;
    int64_t tile, tile_end, tile_step;
    if (MODE == MODE_FILTER) {
        tile = (int64_t)blockIdx.x * kScanWaves + wave;
        tile_step = (int64_t)gridDim.x * kScanWaves;
        tile_end = n_tiles_all;
    } else {
        const int64_t tile0 = (int64_t)blockIdx.x * tiles_per_wave * kScanWaves;
        if (tile0 >= n_tiles_all) return;
        tile = tile0 + wave;
        tile_step = kScanWaves;
        tile_end = tile0 + (int64_t)tiles_per_wave * kScanWaves;
        if (tile_end > n_tiles_all) tile_end = n_tiles_all;
    }

    // operand A: lane (j, m) holds the code chunk 4 s + j of head m % 4 (zero for missing heads)
    i32x4 qa[KS];
    {
        const int j = lane >> 4, r = lane & 3;
        const i32x4* p = reinterpret_cast<const i32x4*>(bf.q8 + (head0 + (r < G ? r : 0)) * D) + j;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            i32x4 v = p[4 * s];
            if (r >= G) v = i32x4{0, 0, 0, 0};
            qa[s] = v;
        }
    }
    float qs0 = bf.qscale[head0], qs1 = 1 < G ? bf.qscale[head0 + 1] : 0.f, qs2 = 2 < G ? bf.qscale[head0 + 2] : 0.f,
          qs3 = 3 < G ? bf.qscale[head0 + 3] : 0.f;
    const int64_t head_rows = ((int64_t)b * sh.Hkv + kvh) * sh.Ncap;
    const int8_t* Kh = bf.K8 + head_rows * D;
    const float* Sh = bf.Kscale + head_rows;

    const int seg_cap = sh.seg_cap;
    const int sid = (int)blockIdx.x * kScanWaves + wave;
    uint64_t* const list0 = bf.cand + head0 * (int64_t)sh.cand_cap;
    __shared__ uint64_t stage_lds[MODE == MODE_FILTER ? kScanWaves * 4 * kStage : 1];
    uint64_t* const st0 = stage_lds + (MODE == MODE_FILTER ? wave * 4 * kStage : 0);
    CandStage cs0{st0, list0, sid, 0, 0}, cs1{st0 + kStage, list0 + (int64_t)sh.cand_cap, sid, 0, 0},
        cs2{st0 + 2 * kStage, list0 + 2 * (int64_t)sh.cand_cap, sid, 0, 0},
        cs3{st0 + 3 * kStage, list0 + 3 * (int64_t)sh.cand_cap, sid, 0, 0};
    float thr0 = 0.f, thr1 = 0.f, thr2 = 0.f, thr3 = 0.f;
    if (MODE == MODE_FILTER) {
        thr0 = bf.thr[head0];
        if (1 < G) thr1 = bf.thr[head0 + 1];
        if (2 < G) thr2 = bf.thr[head0 + 2];
        if (3 < G) thr3 = bf.thr[head0 + 3];
    }

    auto row_of = [&](int64_t item0, int slot) -> int64_t {
        int64_t p = item0 + slot;
        if (MODE == MODE_SAMPLE) {
            if (p > n_items - 1) p = n_items - 1;
            p = sample_pos((int)p, stride);
        }
        return p < N ? p : N - 1;
    };
    auto consume = [&](const i32x4& res, float ks, int64_t item0) {
        const int64_t item = item0 + lane;
        const bool valid = item < n_items;
        const float s0 = (float)res[0] * (qs0 * ks), s1 = (float)res[1] * (qs1 * ks), s2 = (float)res[2] * (qs2 * ks),
                    s3 = (float)res[3] * (qs3 * ks);
        if (MODE == MODE_SAMPLE || MODE == MODE_FULL) {
            float* out = MODE == MODE_SAMPLE ? bf.samp : dst;
            const int64_t pitch = MODE == MODE_SAMPLE ? (int64_t)sh.samp_cap : sh.Ncap;
            if (valid) {
                out[head0 * pitch + item] = s0;
                if (1 < G) out[(head0 + 1) * pitch + item] = s1;
                if (2 < G) out[(head0 + 2) * pitch + item] = s2;
                if (3 < G) out[(head0 + 3) * pitch + item] = s3;
            }
        } else {
            filter_head(s0, thr0, cs0, valid, item, seg_cap, sh.n_seg);
            if (1 < G) filter_head(s1, thr1, cs1, valid, item, seg_cap, sh.n_seg);
            if (2 < G) filter_head(s2, thr2, cs2, valid, item, seg_cap, sh.n_seg);
            if (3 < G) filter_head(s3, thr3, cs3, valid, item, seg_cap, sh.n_seg);
        }
    };

    i32x4 ba[4][KS], bb[4][KS];
    float ksa, ksb;
    // filter: the wave takes one tile of every row of n_seg tiles (seg_tile()); the walk then counts rows, and a
    // tile of the last row that lies beyond the cache re-reads the last key rows and keeps nothing
    const int n_seg_w = (int)tile_step, sid_w = (int)tile;
    if (MODE == MODE_FILTER) {
        tile = 0;
        tile_step = 1;
        tile_end = (n_tiles_all + n_seg_w - 1) / n_seg_w;
    }
    auto tile_of = [&](int64_t t) -> int64_t { return MODE == MODE_FILTER ? seg_tile(t, sid_w, n_seg_w) : t; };
    if (tile < tile_end) {
        tile_load8<D>(Kh, Sh, [&](int slot) { return row_of(tile_of(tile) * 64, slot); }, ba, ksa);
        while (true) {
            const int64_t t1 = tile + tile_step;
            const int64_t p1 = t1 < tile_end ? t1 : tile;
            tile_load8<D>(Kh, Sh, [&](int slot) { return row_of(tile_of(p1) * 64, slot); }, bb, ksb);
            __builtin_amdgcn_sched_barrier(0);
            consume(tile_mac8<D>(ba, qa), ksa, tile_of(tile) * 64);
            if (t1 >= tile_end) break;
            const int64_t t2 = t1 + tile_step;
            const int64_t p2 = t2 < tile_end ? t2 : t1;
            tile_load8<D>(Kh, Sh, [&](int slot) { return row_of(tile_of(p2) * 64, slot); }, ba, ksa);
            __builtin_amdgcn_sched_barrier(0);
            consume(tile_mac8<D>(bb, qa), ksb, tile_of(t1) * 64);
            if (t2 >= tile_end) break;
            tile = t2;
        }
    }
    if (MODE == MODE_FILTER) {
        stage_flush(cs0, seg_cap, sh.n_seg, true);
        if (1 < G) stage_flush(cs1, seg_cap, sh.n_seg, true);
        if (2 < G) stage_flush(cs2, seg_cap, sh.n_seg, true);
        if (3 < G) stage_flush(cs3, seg_cap, sh.n_seg, true);
        if (lane == 0) {
            uint32_t* sc = bf.seg_cnt + head0 * (int64_t)sh.n_seg + sid;
            sc[0] = (uint32_t)cs0.n_glob;
            if (1 < G) sc[sh.n_seg] = (uint32_t)cs1.n_glob;
            if (2 < G) sc[2 * (int64_t)sh.n_seg] = (uint32_t)cs2.n_glob;
            if (3 < G) sc[3 * (int64_t)sh.n_seg] = (uint32_t)cs3.n_glob;
        }
    }
}

template <int MODE>
static hipError_t launch_scan8(const Shape& s, const Bufs& b, int64_t n_items, float* dst, hipStream_t st) {
    dim3 grid, block(kScanWaves * kWave);
    int tpw = 0;
    if (MODE == MODE_FILTER) {
        grid = dim3((unsigned)(s.n_seg / kScanWaves), (unsigned)s.Hkv, (unsigned)s.B);
    } else {
        tpw = tiles_per_wave_for(n_items, s.B, s.Hkv);
        const int64_t tiles = (n_items + 63) / 64, per_wg = (int64_t)tpw * kScanWaves;
        grid = dim3((unsigned)((tiles + per_wg - 1) / per_wg), (unsigned)s.Hkv, (unsigned)s.B);
    }
    if (s.D == 128) hipLaunchKernelGGL((scan8_kernel<128, MODE>), grid, block, 0, st, s, b, tpw, dst);
    else if (s.D == 64) hipLaunchKernelGGL((scan8_kernel<64, MODE>), grid, block, 0, st, s, b, tpw, dst);
    else if (s.D == 256) hipLaunchKernelGGL((scan8_kernel<256, MODE>), grid, block, 0, st, s, b, tpw, dst);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_scan8_sample(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st) {
    Plan pl = make_plan(Nmax, s.k, 1);
    return launch_scan8<MODE_SAMPLE>(s, b, pl.n_samp, nullptr, st);
}
hipError_t launch_scan8_filter(const Shape& s, const Bufs& b, hipStream_t st) {
    return launch_scan8<MODE_FILTER>(s, b, 0, nullptr, st);
}
hipError_t launch_scan8_full(const Shape& s, const Bufs& b, int64_t Nmax, float* dst, hipStream_t st) {
    return launch_scan8<MODE_FULL>(s, b, Nmax, dst, st);
}

// ---------------------------------------------------------------------------------------
// Exact refinement: the score of every candidate the index scan kept is replaced by the
// fp32 dot product of the query with the 16-bit key row.  One wave per segment of a head's
// candidate list (it knows the segment's length, so no slot is visited in vain), D / 8 lanes
// per candidate, kRerankInFlight candidates in flight per lane group (an entry, then the row
// it points to, are dependent loads).
// ---------------------------------------------------------------------------------------
constexpr int kRerankInFlight = 4;    // the best of 1, 2, 4, 8, 16 measured

template <int DT>
__global__ void __launch_bounds__(256) rerank_kernel(Shape sh, Bufs bf) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    constexpr int U = kRerankInFlight;
    __shared__ float qf[256];
    __shared__ uint32_t hist_lds[kTailBins];             // this workgroup's candidates per score bin (exact scores)
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int g = (int)blockIdx.x * 4 + wave;            // this wave's segment
    uint32_t* hist_out = bf.hist + (bh * sh.hist_cap + blockIdx.x) * kTailBins;
    const bool counts = (int)blockIdx.x < sh.hist_cap;   // (always, when the tail is going to read them)
    if (bf.flags[bh]) {                                  // not filtered: the exact redo scores this head itself
        if (counts && threadIdx.x < kTailBins) hist_out[threadIdx.x] = 0u;
        if (lane == 0) bf.seg_max[bh * sh.n_seg + g] = -INFINITY;
        return;
    }
    const int D = sh.D;
    const int lpr = D / EPL, groups = kWave / lpr;       // 16 lanes per candidate at D = 128: 4 groups per wave
    const int grp = lane / lpr, c = lane % lpr;
    const float bin_lo = bf.bins[2 * bh], bin_inv = bf.bins[2 * bh + 1];
    for (int i = threadIdx.x; i < D; i += 256) {
        const char* qp = static_cast<const char*>(bf.q) + (bh * D + i) * Elem<DT>::kBytes;
        qf[i] = DT == DT_F16 ? (float)*reinterpret_cast<const _Float16*>(qp)
                             : __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(qp) << 16);
    }
    if (threadIdx.x < kTailBins) hist_lds[threadIdx.x] = 0u;
    __syncthreads();
    float qr[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) qr[e] = qf[c * EPL + e];
    uint32_t have = bf.seg_cnt[bh * sh.n_seg + g];
    if (have > (uint32_t)sh.seg_cap) have = (uint32_t)sh.seg_cap;
    const char* Kh = static_cast<const char*>(bf.K) +
                     ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * D * Elem<DT>::kBytes;
    uint64_t* list = bf.cand + bh * (int64_t)sh.cand_cap;
    float top = -INFINITY;                               // largest exact score of the segment
    for (uint32_t e0 = 0; e0 < have; e0 += groups * U) {          // `have` is uniform over the wave
        bool ok[U];
        int64_t slot[U];
        uint64_t ent[U];
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t e = e0 + groups * u + grp;
            ok[u] = e < have;
            slot[u] = cand_slot(ok[u] ? e : 0, g, sh.n_seg);
            ent[u] = ok[u] ? list[slot[u]] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            raw[u] = *reinterpret_cast<const u32x4*>(Kh + ((int64_t)(uint32_t)ent[u] * D + c * EPL) * Elem<DT>::kBytes);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
            Elem<DT>::widen(raw[u], kf);
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc = fmaf(kf[i], qr[i], acc);
            for (int o = 1; o < lpr; o <<= 1) acc += wave_xor(acc, o);
            if (ok[u] && c == 0) {
                const float sc = acc + 0.0f;
                list[slot[u]] = ((uint64_t)__float_as_uint(sc) << 32) | (ent[u] & 0xFFFFFFFFull);
                atomicAdd(&hist_lds[tail_bin(sc, bin_lo, bin_inv)], 1u);
                top = fmaxf(top, sc);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) top = fmaxf(top, wave_xor(top, o));
    if (lane == 0) bf.seg_max[bh * sh.n_seg + g] = top;
    __syncthreads();
    if (counts && threadIdx.x < kTailBins) hist_out[threadIdx.x] = hist_lds[threadIdx.x];
}

hipError_t launch_rerank(const Shape& s, const Bufs& b, hipStream_t st) {
    dim3 grid((unsigned)(s.n_seg / 4), (unsigned)s.Hq, (unsigned)s.B);      // n_seg is a multiple of 4
    if (s.dtype == DT_F16) hipLaunchKernelGGL((rerank_kernel<DT_F16>), grid, dim3(256), 0, st, s, b);
    else if (s.dtype == DT_BF16) hipLaunchKernelGGL((rerank_kernel<DT_BF16>), grid, dim3(256), 0, st, s, b);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace tka
