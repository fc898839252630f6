// MFMA tile routines of the key scan over 16-bit keys: operand layouts, tile loads, the
// double-buffered tile walk and the per-tile contraction (used by scan.hip and by the exact
// rescoring in tail.hip).
#pragma once
#include "device_utils.h"
#include "internal.h"

namespace tka {

template <int DT> struct Mfma;
template <> struct Mfma<DT_F16> {
    using v8 = f16x8;
    static __device__ __forceinline__ f32x4 mac(v8 a, v8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma<DT_BF16> {
    using v8 = bf16x8;
    static __device__ __forceinline__ f32x4 mac(v8 a, v8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

// Query block of the group in operand-A layout: lane (j, m) holds channels
// 32 s + 8 j .. +7 of head m % 4 (zero for heads the group does not have).
template <int DT, int D>
__device__ __forceinline__ void load_query_a(const void* q, int64_t head0, int G,
                                             typename Mfma<DT>::v8 (&qa)[D / 32]) {
    using v8 = typename Mfma<DT>::v8;
    const int lane = lane_id();
    const int j = lane >> 4, r = lane & 3;
    const v8* p = reinterpret_cast<const v8*>(static_cast<const char*>(q) + (head0 + (r < G ? r : 0)) * D * 2) + j;
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        v8 v = p[4 * s];
        if (r >= G) v = v8{};
        qa[s] = v;
    }
}

// Operand B of a 64-key tile: for each 16-key sub-tile g, lane (j, n) loads the 16-byte
// chunks 4 s + j (s = 0 .. D/32-1) of the row rowfn(16 g + n).  All loads are issued
// before anything consumes them.
template <int DT, int D, class RowFn>
__device__ __forceinline__ void tile_load(const char* Kh, RowFn rowfn, typename Mfma<DT>::v8 (&b)[4][D / 32]) {
    using v8 = typename Mfma<DT>::v8;
    constexpr int KS = D / 32;
    const int lane = lane_id();
    const int j = lane >> 4, n = lane & 15;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t row = rowfn(16 * g + n);
        const v8* p = reinterpret_cast<const v8*>(Kh + row * (D * 2)) + j;
#pragma unroll
        for (int s = 0; s < KS; ++s) b[g][s] = p[4 * s];
    }
}

// The same for a tile whose 64 rows all exist, through buffer loads: the tile's address
// (wave-uniform) sits in a scalar buffer descriptor, the 16-row sub-tile is a scalar offset
// and lane_off = (n * D + 8 j) * 2 the lane's loop-invariant byte offset, so the loop holds
// no per-lane address arithmetic at all.  (With per-lane 64-bit addresses the compiler
// builds them in registers of the buffer it is about to refill and then waits for every
// outstanding load before it may overwrite them, which serialises every other prefetch.)
template <int DT, int D>
__device__ __forceinline__ void tile_load_full(const char* tile_base, uint32_t lane_off,
                                               typename Mfma<DT>::v8 (&b)[4][D / 32]) {
    using v8 = typename Mfma<DT>::v8;
    constexpr int KS = D / 32;
    // raw buffer (stride 0), 64 * D * 2 bytes long, 32-bit data format
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(tile_base), 0, 64 * D * 2, 0x00020000);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_off + 64 * s, g * 16 * D * 2, 0);
            b[g][s] = __builtin_bit_cast(v8, v);
        }
    }
}

// A wave's walk over the tiles tile, tile + step, ... < end with two register buffers: the
// next tile's loads are in flight while the current one is multiplied and filtered.  The
// prefetch is unconditional (past the end it re-reads a tile the wave already had, a cache
// hit) so that the wait before the MFMAs only covers the tile they consume.  Returns the
// first tile of the sequence at or past `end`.
template <bool PIPELINED, class Buf, class Load, class Use>
__device__ __forceinline__ int64_t walk_tiles(int64_t tile, int64_t end, int64_t step, Buf& ba, Buf& bb, Load load,
                                              Use use) {
  if (PIPELINED) {
    if (tile < end) {
        load(ba, tile);
        while (true) {
            const int64_t t1 = tile + step;
            load(bb, t1 < end ? t1 : tile);
            __builtin_amdgcn_sched_barrier(0);
            use(ba, tile);
            if (t1 >= end) { tile = t1; break; }
            const int64_t t2 = t1 + step;
            load(ba, t2 < end ? t2 : t1);
            __builtin_amdgcn_sched_barrier(0);
            use(bb, t1);
            if (t2 >= end) { tile = t2; break; }
            tile = t2;
        }
    }
  } else {       // one buffer: the other waves of the compute unit cover the latency
    for (; tile < end; tile += step) {
        load(ba, tile);
        __builtin_amdgcn_sched_barrier(0);
        use(ba, tile);
    }
  }
    return tile;
}

// head_dim 256 makes a 64-key tile 32 KiB: two register buffers of it do not fit, and
// with 8 waves per compute unit 256 KiB are in flight anyway.
template <int D> struct ScanPipelined { static constexpr bool value = D <= 128; };

// Scores of the tile: lane l gets res[r] = q_{head0 + r} . K[row(l)].
template <int DT, int D>
__device__ __forceinline__ f32x4 tile_mac(const typename Mfma<DT>::v8 (&b)[4][D / 32],
                                          const typename Mfma<DT>::v8 (&qa)[D / 32]) {
    constexpr int KS = D / 32;
    const int j = lane_id() >> 4;
    f32x4 c[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        c[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) c[g] = Mfma<DT>::mac(qa[s], b[g][s], c[g]);
    }
    // rows 4 jj .. 4 jj + 3 of every accumulator hold heads 0..3; lane group jj keeps sub-tile jj
    f32x4 res;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float lo = (j & 1) ? c[1][r] : c[0][r];
        const float hi = (j & 1) ? c[3][r] : c[2][r];
        res[r] = (j & 2) ? hi : lo;
    }
    return res;
}

}  // namespace tka
