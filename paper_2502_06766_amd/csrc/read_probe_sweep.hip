// Measurement program (not part of the library): how fast can plain 128-bit loads stream 2 GiB out of
// HBM on this GPU, over the launch shapes a key scan could take?  The key scan of the decode path is a
// streaming read of the keys with a little arithmetic per tile, so the best figure here is its ceiling.
//
// Shapes: waves per workgroup (4, 8), workgroups per compute unit (1, 2, 4), bytes a wave has in flight
// (8, 16, 32 KiB: one batch of loads, or two batches double-buffered), and the tile -> wave mapping:
//   strided        wave w of all takes tiles w, w + n_waves, ...            (what the key scan does)
//   wave-range     every wave owns one contiguous range of tiles
//   wg-range       every workgroup owns a contiguous range, its waves interleaved
//   xcd-range      workgroup b runs on XCD b % 8: each XCD owns one contiguous eighth of the buffer
//   xcd-cyclic B   blocks of B tiles go to the XCDs round-robin, strided inside an XCD
// Four distinct 2 GiB buffers are read in turn, so nothing is found in a cache.  Prints a markdown table
// (median and best of 8 timed launches after 2 warm-up launches, HIP events around each launch).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x)                                                                       \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            exit(1);                                                                \
        }                                                                           \
    } while (0)

enum { STRIDED = 0, WAVE_RANGE = 1, WG_RANGE = 2, XCD_RANGE = 3, XCD_CYCLIC = 4 };

// A tile is LOADS * 1 KiB: every lane loads LOADS 16-byte words, 1 KiB apart.
template <int WAVES, int LOADS, bool DOUBLE, int ORDER, int BLK>
__global__ void __launch_bounds__(WAVES * 64) read_kernel(const u32x4* __restrict__ src, size_t n_tiles, uint32_t* sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t n_waves = (size_t)gridDim.x * WAVES, w_all = (size_t)blockIdx.x * WAVES + wave;
    size_t tile = 0, step = 1, end = 0;
    if (ORDER == STRIDED) { tile = w_all; step = n_waves; end = n_tiles; }
    if (ORDER == WAVE_RANGE) {
        const size_t per = (n_tiles + n_waves - 1) / n_waves;
        tile = w_all * per; end = std::min(n_tiles, tile + per);
    }
    if (ORDER == WG_RANGE) {
        const size_t per = (n_tiles + gridDim.x - 1) / gridDim.x;
        tile = (size_t)blockIdx.x * per + wave; step = WAVES; end = std::min(n_tiles, (size_t)blockIdx.x * per + per);
    }
    const size_t xcd = blockIdx.x & 7, per_xcd = n_tiles / 8;                  // (grids are multiples of 8)
    const size_t w_xcd = (size_t)(blockIdx.x >> 3) * WAVES + wave, waves_xcd = (size_t)(gridDim.x >> 3) * WAVES;
    if (ORDER == XCD_RANGE) { tile = xcd * per_xcd + w_xcd; step = waves_xcd; end = xcd * per_xcd + per_xcd; }
    if (ORDER == XCD_CYCLIC) { tile = w_xcd; step = waves_xcd; end = per_xcd; }
    uint32_t acc = 0;
    u32x4 a[LOADS], b[LOADS];
    auto load = [&](u32x4(&v)[LOADS], size_t t) {
        if (ORDER == XCD_CYCLIC) t = ((t / BLK) * 8 + xcd) * BLK + t % BLK;     // the t-th tile of this XCD
        const u32x4* p = src + t * (LOADS * 64) + lane;
#pragma unroll
        for (int u = 0; u < LOADS; ++u) v[u] = p[u * 64];
    };
    auto use = [&](u32x4(&v)[LOADS]) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    };
    if (DOUBLE) {
        if (tile < end) {
            load(a, tile);
            while (true) {
                const size_t t1 = tile + step;
                load(b, t1 < end ? t1 : tile);
                __builtin_amdgcn_sched_barrier(0);
                use(a);
                if (t1 >= end) break;
                const size_t t2 = t1 + step;
                load(a, t2 < end ? t2 : t1);
                __builtin_amdgcn_sched_barrier(0);
                use(b);
                if (t2 >= end) break;
                tile = t2;
            }
        }
    } else {
        for (; tile < end; tile += step) {
            load(a, tile);
            __builtin_amdgcn_sched_barrier(0);
            use(a);
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;        // keeps the loads alive
}

static std::vector<char*> g_bufs;
static uint32_t* g_sink;
static int g_cu;
static const size_t kBytes = (size_t)2 << 30;

template <int WAVES, int LOADS, bool DOUBLE, int ORDER, int BLK = 1>
static void run(const char* mapping, int wgs_per_cu) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const size_t n_tiles = kBytes / ((size_t)LOADS * 1024);
    std::vector<float> ms;
    for (int it = 0; it < 10; ++it) {
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL((read_kernel<WAVES, LOADS, DOUBLE, ORDER, BLK>), dim3(g_cu * wgs_per_cu), dim3(WAVES * 64), 0, 0,
                           (const u32x4*)g_bufs[it % g_bufs.size()], n_tiles, g_sink);
        CK(hipGetLastError());
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float t;
        CK(hipEventElapsedTime(&t, e0, e1));
        if (it >= 2) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    printf("| %d | %d | %s%d KiB | %s | %.0f | %.0f | %.1f |\n", WAVES, wgs_per_cu, DOUBLE ? "2 x " : "", LOADS, mapping,
           kBytes / ms[ms.size() / 2] / 1e6, kBytes / ms[0] / 1e6, ms[ms.size() / 2] * 1e3);
    fflush(stdout);
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
}

int main() {
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    g_cu = p.multiProcessorCount;
    if (g_cu % 8) { printf("expected a multiple of 8 compute units\n"); return 1; }
    printf("device %s, %d compute units; 2 GiB per launch, 4 buffers in turn\n\n", p.name, g_cu);
    g_bufs.resize(4);
    for (auto& b : g_bufs) {
        CK(hipMalloc(&b, kBytes));
        CK(hipMemset(b, 1, kBytes));
    }
    CK(hipMalloc(&g_sink, 4096));
    CK(hipDeviceSynchronize());
    printf("| waves/wg | wgs/CU | in flight per wave | mapping | median GB/s | best GB/s | median us |\n|---|---|---|---|---|---|---|\n");
    // workgroups per compute unit x bytes in flight, strided mapping
    run<4, 8, false, STRIDED>("strided", 1);
    run<4, 8, false, STRIDED>("strided", 2);
    run<4, 8, false, STRIDED>("strided", 4);
    run<4, 16, false, STRIDED>("strided", 1);
    run<4, 16, false, STRIDED>("strided", 2);
    run<4, 16, false, STRIDED>("strided", 4);
    run<4, 32, false, STRIDED>("strided", 1);
    run<4, 32, false, STRIDED>("strided", 2);
    run<4, 8, true, STRIDED>("strided", 1);
    run<4, 8, true, STRIDED>("strided", 2);
    run<4, 8, true, STRIDED>("strided", 4);
    run<4, 16, true, STRIDED>("strided", 1);
    run<4, 16, true, STRIDED>("strided", 2);
    run<8, 8, true, STRIDED>("strided", 1);
    run<8, 8, true, STRIDED>("strided", 2);
    run<8, 16, true, STRIDED>("strided", 1);
    // mappings at the key scan's shape (4 waves, 2 workgroups per compute unit, 2 x 16 KiB)
    run<4, 16, true, WAVE_RANGE>("wave-range", 2);
    run<4, 16, true, WG_RANGE>("wg-range", 2);
    run<4, 16, true, XCD_RANGE>("xcd-range", 2);
    run<4, 16, true, XCD_CYCLIC, 1>("xcd-cyclic 16 KiB", 2);
    run<4, 16, true, XCD_CYCLIC, 16>("xcd-cyclic 256 KiB", 2);
    run<4, 16, true, XCD_CYCLIC, 128>("xcd-cyclic 2 MiB", 2);
    run<4, 16, true, XCD_CYCLIC, 2048>("xcd-cyclic 32 MiB", 2);
    run<8, 16, true, XCD_RANGE>("xcd-range", 1);
    run<8, 16, true, XCD_CYCLIC, 128>("xcd-cyclic 2 MiB", 1);
    // the first shape again: drift over the run
    run<4, 16, true, STRIDED>("strided (again)", 2);
    return 0;
}
