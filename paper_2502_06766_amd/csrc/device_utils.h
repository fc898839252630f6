// Device-side helpers for the gfx950 kernels (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tka {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

// Monotone map float -> uint32: a < b  <=>  ord(a) < ord(b) (for non-NaN; -0 is
// canonicalised to +0 by the caller adding 0.0f).
__device__ __forceinline__ uint32_t ord_from_bits(uint32_t u) {
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ uint32_t bits_from_ord(uint32_t o) {
    return o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu);
}
// Orders this wave's LDS/global accesses as seen by its own lanes.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// number of set bits of `m` below this lane
__device__ __forceinline__ int mask_rank(uint64_t m) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

template <typename T>
__device__ __forceinline__ T wave_xor(T v, int mask) {
    return __shfl_xor(v, mask, 64);
}

// widen the 16 bytes a lane loaded into fp32 values
template <int DT> struct Elem;
template <> struct Elem<0> {  // fp32
    static constexpr int kBytes = 4, kPerLoad = 4;
    static __device__ __forceinline__ void widen(const u32x4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct Elem<1> {  // fp16
    static constexpr int kBytes = 2, kPerLoad = 8;
    static __device__ __forceinline__ void widen(const u32x4& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            union { uint32_t u; _Float16 h[2]; } cv;
            cv.u = w[i];
            f[2 * i] = (float)cv.h[0];
            f[2 * i + 1] = (float)cv.h[1];
        }
    }
};
template <> struct Elem<2> {  // bf16
    static constexpr int kBytes = 2, kPerLoad = 8;
    static __device__ __forceinline__ void widen(const u32x4& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

}  // namespace tka
