// Host-side walk through the C ABI for the sanitizer run (tests/test_sanitizers_cpu.py):
// api.hip is linked with stand-ins for the kernel launchers of the other translation units,
// and only calls that need no device (sizes, schedules, argument checks) or that fail before
// touching one are made.  Every check that fails prints a line and makes the exit status 1.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "../include/topk_attn.h"
#include "../include/topk_attn_debug.h"
#include "../paper_2502_06766_amd/csrc/internal.h"

namespace tka {
// never reached: no handle is ever created in this program
hipError_t launch_scan_sample(const Shape&, const Bufs&, int64_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_scan_filter(const Shape&, const Bufs&, int64_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_scan_full(const Shape&, const Bufs&, int64_t, float*, hipStream_t) { return hipErrorUnknown; }
bool scan_mfma_supported(const Shape&) { return false; }
hipError_t launch_threshold(const Shape&, const Bufs&, int64_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_select_full(const Shape&, const Bufs&, int64_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_gather(const Shape&, const Bufs&, hipStream_t) { return hipErrorUnknown; }
bool tail_supported(const Shape&) { return false; }
hipError_t launch_tail(const Shape&, const Bufs&, hipStream_t) { return hipErrorUnknown; }
bool index8_supported(int dtype, int D, int G) { return dtype != 0 && D >= 64 && G <= 4; }
bool pages_supported(int dtype, int, int G) { return dtype != 0 && G <= 4; }
hipError_t launch_page_balls(int, int, const void*, int64_t, int64_t, int, int, const int32_t*, int64_t, int64_t, void*, float*,
                             hipStream_t) {
    return hipErrorUnknown;
}
hipError_t launch_page_filter(const Shape&, const Bufs&, float, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_scan_filter_paged(const Shape&, const Bufs&, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_quantize_rows(int, int, const void*, int64_t, int64_t, int, int8_t*, float*, int64_t, hipStream_t) {
    return hipErrorUnknown;
}
hipError_t launch_append_step_small8(int, int, const void*, const void*, void*, void*, int64_t, int, int64_t, int, int64_t,
                                     int32_t*, int8_t*, float*, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_quantize_step(int, int, const void*, int, int64_t, int, int64_t, const int32_t*, int8_t*, float*,
                                hipStream_t) {
    return hipErrorUnknown;
}
hipError_t launch_scan8_sample(const Shape&, const Bufs&, int64_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_scan8_filter(const Shape&, const Bufs&, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_scan8_full(const Shape&, const Bufs&, int64_t, float*, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_rerank(const Shape&, const Bufs&, hipStream_t) { return hipErrorUnknown; }
}  // namespace tka

static int failures = 0;
#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            printf("abi driver: line %d: %s\n", __LINE__, #cond);        \
            ++failures;                                                  \
        }                                                                \
    } while (0)

static topk_attn_config base_config() {
    topk_attn_config c;
    memset(&c, 0, sizeof c);
    c.struct_size = sizeof c;
    c.n_layers = 2; c.n_seqs = 3; c.n_q_heads = 32; c.n_kv_heads = 8; c.head_dim = 128;
    c.max_tokens = 100000; c.max_k = 2048; c.dtype = TOPK_ATTN_F16; c.device = 0;
    return c;
}

int main() {
    // sizes
    topk_attn_config c = base_config();
    const size_t kv = topk_attn_kv_bytes(&c), ws = topk_attn_workspace_bytes(&c);
    CHECK(kv == 2ull * 2 * 3 * 8 * 100000 * 128 * 2);
    CHECK(ws > 0);
    c.index_kind = TOPK_ATTN_INDEX_INT8;
    CHECK(topk_attn_kv_bytes(&c) > kv);
    c.index_kind = 9;
    CHECK(topk_attn_kv_bytes(&c) == 0 && topk_attn_workspace_bytes(&c) == 0);
    CHECK(topk_attn_kv_bytes(nullptr) == 0 && topk_attn_workspace_bytes(nullptr) == 0);
    // the largest configurations the checks let through must not overflow the size arithmetic
    c = base_config();
    c.n_layers = 128; c.n_seqs = 64; c.max_tokens = 0x7FFFFF00ll; c.max_k = 1 << 28; c.max_window = 0x7FFFFFFF;
    c.max_queries = 1;
    CHECK(topk_attn_kv_bytes(&c) > 0 && topk_attn_workspace_bytes(&c) > 0);
    // every field out of range once
    topk_attn_t* h = reinterpret_cast<topk_attn_t*>(0x1);
    struct { int field; int64_t value; int want; } bad[] = {
        {0, 0, TOPK_ATTN_EINVAL}, {1, 0, TOPK_ATTN_EINVAL}, {2, 30, TOPK_ATTN_EUNSUPPORTED},
        {3, 96, TOPK_ATTN_EUNSUPPORTED}, {4, 0, TOPK_ATTN_EINVAL}, {4, 1ll << 31, TOPK_ATTN_EINVAL},
        {5, 0, TOPK_ATTN_EINVAL}, {6, 7, TOPK_ATTN_EUNSUPPORTED}, {7, -1, TOPK_ATTN_EINVAL},
        {8, -1, TOPK_ATTN_EINVAL}, {9, 5000, TOPK_ATTN_EINVAL}, {10, 3, TOPK_ATTN_EINVAL},
        {5, (1 << 28) + 1, TOPK_ATTN_EINVAL},
    };
    for (auto& b : bad) {
        c = base_config();
        switch (b.field) {
            case 0: c.n_layers = (int)b.value; break;
            case 1: c.n_seqs = (int)b.value; break;
            case 2: c.n_q_heads = (int)b.value; break;
            case 3: c.head_dim = (int)b.value; break;
            case 4: c.max_tokens = b.value; break;
            case 5: c.max_k = (int)b.value; break;
            case 6: c.dtype = (int)b.value; break;
            case 7: c.device = (int)b.value; break;
            case 8: c.max_window = (int)b.value; break;
            case 9: c.max_queries = (int)b.value; break;
            case 10: c.index_kind = (int)b.value; break;
        }
        h = reinterpret_cast<topk_attn_t*>(0x1);
        CHECK(topk_attn_create(&c, &h) == b.want);
        CHECK(h == nullptr);
        CHECK(topk_attn_kv_bytes(&c) == 0);
    }
    c = base_config();
    CHECK(topk_attn_create(&c, &h) == TOPK_ATTN_EINVAL && h == nullptr);       // null storage
    CHECK(topk_attn_create(&c, nullptr) == TOPK_ATTN_EINVAL);
    c.kv_storage = reinterpret_cast<void*>(0x1000); c.workspace = reinterpret_cast<void*>(0x2010);
    c.kv_bytes = kv; c.workspace_bytes = ws;
    CHECK(topk_attn_create(&c, &h) == TOPK_ATTN_EINVAL);                        // misaligned workspace
    c.workspace = reinterpret_cast<void*>(0x2000); c.workspace_bytes = ws - 1;
    CHECK(topk_attn_create(&c, &h) == TOPK_ATTN_ENOMEM && h == nullptr);       // buffer too small
    c.struct_size = 12;
    CHECK(topk_attn_create(&c, &h) == TOPK_ATTN_EINVAL);
    // no device is visible to this program: a valid configuration fails cleanly and frees its handle
    c = base_config();
    c.kv_storage = reinterpret_cast<void*>(0x1000); c.workspace = reinterpret_cast<void*>(0x2000);
    c.kv_bytes = kv; c.workspace_bytes = ws;
    CHECK(topk_attn_create(&c, &h) == TOPK_ATTN_EDEVICE && h == nullptr);

    // null handles
    float f = 0.f; int n = 0; double ms = 0.0; int32_t k1 = 1;
    CHECK(topk_attn_decode(nullptr, 0, &f, 1, &f, nullptr, nullptr, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_decode_static(nullptr, 0, &f, 1, &f, nullptr, nullptr, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_decode_window(nullptr, 0, &f, 1, 0, &f, nullptr, nullptr, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_decode_multi(nullptr, 0, &f, 2, 1, 1, 0, &f, nullptr, nullptr, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_decode_layers(nullptr, 0, 1, &f, &k1, 0, &f, nullptr, nullptr, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_append_kv(nullptr, 0, 0, &f, &f, 1, 1, 1, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_append_step(nullptr, 0, &f, &f, 1, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_length(nullptr, 0, 0) == -1);
    CHECK(topk_attn_reset(nullptr, 0, 0, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_set_path(nullptr, 0) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_scores(nullptr, 0, &f, &f, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_last_fallbacks(nullptr, &n) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_set_scan_timing(nullptr, 1) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_debug_force_redo(nullptr, 1) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_set_page_bound_scale(nullptr, 1.0f) == TOPK_ATTN_EINVAL);
    { int64_t a = 0, bb = 0; CHECK(topk_attn_last_pages_read(nullptr, &a, &bb) == TOPK_ATTN_EINVAL); }
    c = base_config();
    c.index_kind = TOPK_ATTN_INDEX_PAGES;
    {   // centres and (radius, centre norm) pairs of ceil(100000 / 64) pages per key stream, each region rounded up to 256 bytes
        const unsigned long long pages = 2ull * 3 * 8 * ((100000 + 63) / 64);
        CHECK(topk_attn_kv_bytes(&c) == kv + (pages * 128 * 2 + 255) / 256 * 256 + (pages * 8 + 255) / 256 * 256);
    }
    CHECK(topk_attn_scan_time(nullptr, &ms, &n) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_read_probe(nullptr, 16, nullptr, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_destroy(nullptr) == TOPK_ATTN_EINVAL);
    for (int code = -2; code < 12; ++code) CHECK(strlen(topk_attn_strerror(code)) > 0);
    CHECK(strlen(topk_attn_build_id()) > 0);

    // layer-wise k schedule: budgets, layer counts and ratios over their whole range
    const double ratios[] = {1e-6, 0.25, 0.5, 1.0, 1.5, 3.0, 8.0, 1e6};
    for (int L = 1; L <= 130; L += (L < 8 ? 1 : 17)) {
        std::vector<int32_t> ks((size_t)L);
        for (double r : ratios) {
            for (int64_t total : {(int64_t)L, (int64_t)L + 1, (int64_t)7 * L + 3, (int64_t)8192 * L, (int64_t)INT32_MAX}) {
                const int rc = topk_attn_k_schedule(total, L, r, ks.data());
                if (rc != TOPK_ATTN_OK) {      // only a share beyond int32 may be refused
                    CHECK(total == INT32_MAX && L == 1 ? false : total >= (int64_t)INT32_MAX / 2);
                    continue;
                }
                int64_t sum = 0;
                for (int32_t v : ks) { CHECK(v >= 1); sum += v; }
                CHECK(sum == total);
            }
        }
    }
    int32_t four[4];
    CHECK(topk_attn_k_schedule(3, 4, 1.0, four) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(100, 0, 1.0, four) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(100, 4, 0.0, four) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(100, 4, NAN, four) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(100, 4, INFINITY, four) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(100, 4, 1.0, nullptr) == TOPK_ATTN_EINVAL);
    CHECK(topk_attn_k_schedule(10, 4, 1.0, four) == TOPK_ATTN_OK && four[0] == 2 && four[1] == 2 && four[2] == 3 &&
          four[3] == 3);

    if (failures == 0) printf("abi driver: all checks passed\n");
    return failures ? 1 : 0;
}
