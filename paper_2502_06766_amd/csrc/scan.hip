// Key-scoring scan: S[h, i] = q_h . K[g(h), i] over the cached keys of one layer
// (the score matrix S = q K^T of Eq. 1 of arXiv 2502.06766, raw dot products as used by
// the paper's k-nearest-neighbour search under the dot-product metric).
//
// 16-bit caches use v_mfma_f32_16x16x32_{f16,bf16}: one wave scores a tile of 64
// consecutive keys against the (up to 4) query heads that share the KV head, fp32
// accumulate.  Operand B is loaded straight from the row-major key rows in its MFMA
// register layout (lane (j, n) holds 8 consecutive channels of key n), operand A holds the
// query block replicated in every group of four rows, so that after four accumulators
// (one per 16-key sub-tile) lane l owns the scores of key l for all heads of the group.
//
// Three uses of the same tile routine:
//   sample : score a strided, jittered sample of positions (threshold estimate)
//   filter : score every key, keep (score, position) pairs >= a per-head threshold; every
//            wave appends to a private segment of the head's candidate list (plain stores,
//            no atomics, so the list order is fixed by the launch geometry alone) and the
//            workgroup counts what it kept per score bin for the selection that follows; with
//            a page index the wave reads only the tiles (pages) the index could not rule out
//   full   : score every key and store the fp32 scores
// fp32 caches go through a plain FMA kernel (full only).
#include <type_traits>

#include "device_utils.h"
#include "internal.h"
#include "scan_common.h"
#include "scan_tiles.h"

namespace tka {

// PAGED (filter mode only): the wave skips the tiles whose bit in the page mask is clear (pages of 64 keys
// that the coarse page index has ruled out for every head of the group).
template <int DT, int D, int MODE, bool PAGED = false>
__global__ void __launch_bounds__(kScanWaves* kWave)
scan_mfma_kernel(Shape sh, Bufs bf, int tiles_per_wave, float* dst) {
    using v8 = typename Mfma<DT>::v8;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int G = sh.G;
    const int64_t head0 = (int64_t)b * sh.Hq + (int64_t)kvh * G;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform
    const int64_t N = prefix_len(bf.len[b], sh.window);

    int64_t n_items = N;   // keys (or samples) this (b, kv head) has
    int stride = 1;
    if (MODE == MODE_SAMPLE) {
        if (N == 0) return;          // nothing to search: the whole sequence is inside the window
        Plan pl = make_plan(N, sh.k < N ? sh.k : (int)N);
        n_items = pl.n_samp;
        stride = pl.stride;
    }
    // tiles of this wave.  sample/full: a workgroup owns a contiguous run of tiles and its
    // waves take them round-robin.  filter: wave-segment sid = 4 blockIdx.x + wave takes one tile
    // of every row of n_seg tiles (seg_tile()), so that any clustering of high scores along the
    // sequence spreads evenly over the segments.
    const int64_t n_tiles_all = (n_items + 63) / 64;
    int64_t tile, tile_end, tile_step;
    if (MODE == MODE_FILTER) {
        tile = (int64_t)blockIdx.x * kScanWaves + wave;
        tile_step = (int64_t)gridDim.x * kScanWaves;
        tile_end = n_tiles_all;
    } else {
        const int64_t tile0 = (int64_t)blockIdx.x * tiles_per_wave * kScanWaves;
        if (tile0 >= n_tiles_all) return;   // whole workgroup past the end
        tile = tile0 + wave;
        tile_step = kScanWaves;
        tile_end = tile0 + (int64_t)tiles_per_wave * kScanWaves;
        if (tile_end > n_tiles_all) tile_end = n_tiles_all;
    }

    v8 qa[D / 32];
    load_query_a<DT, D>(bf.q, head0, G, qa);
    const char* Kh = static_cast<const char*>(bf.K) + ((int64_t)b * sh.Hkv + kvh) * sh.Ncap * (D * 2);

    // filter: this wave's segment in each head's candidate list
    const int seg_cap = sh.seg_cap;
    const int sid = (int)blockIdx.x * kScanWaves + wave;
    uint64_t* const list0 = bf.cand + head0 * (int64_t)sh.cand_cap;
    __shared__ uint64_t stage_lds[MODE == MODE_FILTER ? kScanWaves * 4 * kStage : 1];
    uint64_t* const st0 = stage_lds + (MODE == MODE_FILTER ? wave * 4 * kStage : 0);
    CandStage cs0{st0, list0, sid, 0, 0}, cs1{st0 + kStage, list0 + (int64_t)sh.cand_cap, sid, 0, 0},
        cs2{st0 + 2 * kStage, list0 + 2 * (int64_t)sh.cand_cap, sid, 0, 0},
        cs3{st0 + 3 * kStage, list0 + 3 * (int64_t)sh.cand_cap, sid, 0, 0};
    float thr0 = 0.f, thr1 = 0.f, thr2 = 0.f, thr3 = 0.f;
    float lo0 = 0.f, lo1 = 0.f, lo2 = 0.f, lo3 = 0.f, iw0 = 0.f, iw1 = 0.f, iw2 = 0.f, iw3 = 0.f;   // tail_bin() of each head
    float top0 = -INFINITY, top1 = -INFINITY, top2 = -INFINITY, top3 = -INFINITY;   // largest score seen per head
    // candidates of this workgroup per score bin and head (the tail sorts them by bin)
    __shared__ uint32_t hist_lds[MODE == MODE_FILTER ? 4 * kTailBins : 1];
    if (MODE == MODE_FILTER) {
        const float* bins = bf.bins + 2 * head0;
        thr0 = bf.thr[head0]; lo0 = bins[0]; iw0 = bins[1];
        if (1 < G) { thr1 = bf.thr[head0 + 1]; lo1 = bins[2]; iw1 = bins[3]; }
        if (2 < G) { thr2 = bf.thr[head0 + 2]; lo2 = bins[4]; iw2 = bins[5]; }
        if (3 < G) { thr3 = bf.thr[head0 + 3]; lo3 = bins[6]; iw3 = bins[7]; }
        for (int i = threadIdx.x; i < 4 * kTailBins; i += kScanWaves * kWave) hist_lds[i] = 0;
        __syncthreads();
    }

    // row of tile slot `slot` for the tile starting at item `item0`
    auto row_of = [&](int64_t item0, int slot) -> int64_t {
        int64_t p = item0 + slot;
        if (MODE == MODE_SAMPLE) {
            if (p > n_items - 1) p = n_items - 1;
            p = sample_pos((int)p, stride);
        }
        return p < N ? p : N - 1;
    };
    auto consume = [&](const f32x4& res, int64_t item0) {
        const int64_t item = item0 + lane;
        const bool valid = item < n_items;
        if (MODE == MODE_SAMPLE) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (r < G && valid) bf.samp[(head0 + r) * sh.samp_cap + item] = res[r];
        } else if (MODE == MODE_FULL) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (r < G && valid) dst[(head0 + r) * sh.Ncap + item] = res[r];
        } else {
            if (valid) {
                top0 = fmaxf(top0, res[0]); top1 = fmaxf(top1, res[1]);
                top2 = fmaxf(top2, res[2]); top3 = fmaxf(top3, res[3]);
            }
            if (0 < G) filter_head(res[0], thr0, cs0, valid, item, seg_cap, sh.n_seg, hist_lds, lo0, iw0);
            if (1 < G) filter_head(res[1], thr1, cs1, valid, item, seg_cap, sh.n_seg, hist_lds + kTailBins, lo1, iw1);
            if (2 < G) filter_head(res[2], thr2, cs2, valid, item, seg_cap, sh.n_seg, hist_lds + 2 * kTailBins, lo2, iw2);
            if (3 < G) filter_head(res[3], thr3, cs3, valid, item, seg_cap, sh.n_seg, hist_lds + 3 * kTailBins, lo3, iw3);
        }
    };

    struct TileB { v8 b[4][D / 32]; } ba, bb;
    auto load_rows = [&](TileB& t, int64_t ti) { tile_load<DT, D>(Kh, [&](int slot) { return row_of(ti * 64, slot); }, t.b); };
    auto use = [&](TileB& t, int64_t ti) { consume(tile_mac<DT, D>(t.b, qa), ti * 64); };
    if (MODE == MODE_SAMPLE) {
        walk_tiles<ScanPipelined<D>::value>(tile, tile_end, tile_step, ba, bb, load_rows, use);
    } else if (MODE == MODE_FILTER && PAGED) {
        // The pages kept, ascending, are dealt to the wave segments by rank like the tiles of the plain scan
        // (seg_tile() over ranks; 64 rows looked up at a time, one per lane), so every wave reads as many
        // tiles as any other.  They are walked like the plain sequence (next tile's loads in flight
        // while the current one is multiplied and filtered; one buffer at head_dim 256).
        const int64_t stream = (int64_t)b * sh.Hkv + kvh;
        const int32_t* plist = bf.page_list + stream * (int64_t)sh.page_words * 64;
        const int64_t n_kept = (int64_t)bf.page_cnt[stream];
        const int64_t n_whole = N / 64;
        const uint32_t lane_off = (uint32_t)(((lane & 15) * D + (lane >> 4) * 8) * 2);
        const int n_seg = (int)tile_step;
        const int64_t rows = (n_kept + n_seg - 1) / n_seg;      // rows of n_seg ranks; the last one may be short
        int64_t base = 0;                        // first row of the current group of 64
        int32_t mine = 0;                        // lane i: page whose rank is this segment's in row base + i
        uint64_t m = 0ull;                       // rows of the group that hold a page for this segment, not yet taken
        auto look_up = [&]() {
            const int64_t i = base + lane;
            const int64_t r = seg_tile(i, sid, n_seg);
            const bool ok = i < rows && r < n_kept;
            mine = ok ? plist[r] : 0;
            m = __ballot(ok);
        };
        if (rows > 0) look_up();
        auto next = [&]() -> int64_t {           // the wave's next tile to read, or -1 (wave-uniform)
            while (m == 0ull) {
                base += 64;
                if (base >= rows) return -1;
                look_up();
            }
            const int bit = __builtin_ctzll(m);
            m &= m - 1ull;
            return (int64_t)__builtin_amdgcn_readlane(mine, bit);
        };
        auto load_any = [&](TileB& t, int64_t ti) {
            if (ti < n_whole) tile_load_full<DT, D>(Kh + ti * (64 * D * 2), lane_off, t.b);
            else load_rows(t, ti);
        };
        if (rows > 0) {
            int64_t t0 = next();
            if (ScanPipelined<D>::value) {
                if (t0 >= 0) {
                    load_any(ba, t0);
                    while (true) {
                        const int64_t t1 = next();
                        load_any(bb, t1 >= 0 ? t1 : t0);       // past the end: a tile the wave already had
                        __builtin_amdgcn_sched_barrier(0);
                        use(ba, t0);
                        if (t1 < 0) break;
                        const int64_t t2 = next();
                        load_any(ba, t2 >= 0 ? t2 : t1);
                        __builtin_amdgcn_sched_barrier(0);
                        use(bb, t1);
                        if (t2 < 0) break;
                        t0 = t2;
                    }
                }
            } else {
                for (; t0 >= 0; t0 = next()) {
                    load_any(ba, t0);
                    __builtin_amdgcn_sched_barrier(0);
                    use(ba, t0);
                }
            }
        }
    } else {
        if (MODE == MODE_FILTER) {
            // one tile per row of n_seg tiles: the rows made of whole tiles only first, then the last one or two
            // (tiles beyond the cache are skipped, the one its end cuts short is loaded row by row)
            const int n_seg = (int)tile_step;
            const int64_t n_whole = N / 64;
            const int64_t rows_whole = n_whole / n_seg, rows = (n_tiles_all + n_seg - 1) / n_seg;
            const uint32_t lane_off = (uint32_t)(((lane & 15) * D + (lane >> 4) * 8) * 2);
            walk_tiles<ScanPipelined<D>::value>(0, rows_whole, 1, ba, bb,
                [&](TileB& t, int64_t i) { tile_load_full<DT, D>(Kh + seg_tile(i, sid, n_seg) * (64 * D * 2), lane_off, t.b); },
                [&](TileB& t, int64_t i) { use(t, seg_tile(i, sid, n_seg)); });
            for (int64_t i = rows_whole; i < rows; ++i) {
                const int64_t ti = seg_tile(i, sid, n_seg);
                if (ti < n_tiles_all) {
                    load_rows(ba, ti);
                    use(ba, ti);
                }
            }
        } else {
            // whole tiles first, then the one tile (if any) that the end of the cache cuts short
            const int64_t n_whole = N / 64;
            const uint32_t lane_off = (uint32_t)(((lane & 15) * D + (lane >> 4) * 8) * 2);
            tile = walk_tiles<ScanPipelined<D>::value>(tile, tile_end < n_whole ? tile_end : n_whole, tile_step, ba, bb,
                              [&](TileB& t, int64_t ti) { tile_load_full<DT, D>(Kh + ti * (64 * D * 2), lane_off, t.b); }, use);
            for (; tile < tile_end; tile += tile_step) {
                load_rows(ba, tile);
                use(ba, tile);
            }
        }
    }
    if (MODE == MODE_FILTER) {
        stage_flush(cs0, seg_cap, sh.n_seg, true);
        if (1 < G) stage_flush(cs1, seg_cap, sh.n_seg, true);
        if (2 < G) stage_flush(cs2, seg_cap, sh.n_seg, true);
        if (3 < G) stage_flush(cs3, seg_cap, sh.n_seg, true);
        for (int o = 32; o > 0; o >>= 1) {
            top0 = fmaxf(top0, wave_xor(top0, o)); top1 = fmaxf(top1, wave_xor(top1, o));
            top2 = fmaxf(top2, wave_xor(top2, o)); top3 = fmaxf(top3, wave_xor(top3, o));
        }
        if (lane == 0) {
            uint32_t* sc = bf.seg_cnt + head0 * (int64_t)sh.n_seg + sid;
            float* sx = bf.seg_max + head0 * (int64_t)sh.n_seg + sid;
            sc[0] = (uint32_t)cs0.n_glob;
            sx[0] = top0;
            if (1 < G) { sc[sh.n_seg] = (uint32_t)cs1.n_glob; sx[sh.n_seg] = top1; }
            if (2 < G) { sc[2 * (int64_t)sh.n_seg] = (uint32_t)cs2.n_glob; sx[2 * (int64_t)sh.n_seg] = top2; }
            if (3 < G) { sc[3 * (int64_t)sh.n_seg] = (uint32_t)cs3.n_glob; sx[3 * (int64_t)sh.n_seg] = top3; }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < G * kTailBins; i += kScanWaves * kWave)
            bf.hist[((head0 + i / kTailBins) * sh.hist_cap + blockIdx.x) * kTailBins + i % kTailBins] = hist_lds[i];
    }
}

// ---------------------------------------------------------------------------------------
// Row-tile variant: up to 16 (32 with two row tiles) (query, head) rows against one KV head in a single pass over
// its keys -- head groups of 5..16, and several queries per sequence (a chunk of M
// queries, the cache-construction use the paper mentions for top-k attention).  Operand A
// holds 16 distinct rows, so the four accumulators of a 64-key tile give lane (j, n) the
// scores of rows 4 j + i (i = 0..3) for keys n, 16 + n, 32 + n, 48 + n: the same 16 MFMAs
// per tile as the grouped kernel, four times the rows.  Per-row state lives in the 16
// lanes that own the row.  A row's candidates are counted per score bin when they leave
// the row's LDS stage for its segment (the same counts the grouped kernel leaves).
// ---------------------------------------------------------------------------------------
// LDS staging slots per (wave, row): the 64 entries one step can add on top of the remainder
// (fewer than kCandChunk entries) an aligned flush leaves behind
constexpr int kStageRow = 128;
static_assert(kCandChunk <= 16 && kStageRow >= 64 + kCandChunk, "row stage too small for an aligned flush");

// NT row tiles (16 rows each) share every key tile: NT = 2 halves the passes over the keys for
// 17..32 rows at the price of one wave per SIMD (512 registers) and 128 KiB of LDS stages,
// which costs this kernel nothing measurable.
template <int DT, int D, int MODE, int NT>
__global__ void __launch_bounds__(kScanWaves* kWave)
__attribute__((amdgpu_waves_per_eu(NT == 1 ? 2 : 1, NT == 1 ? 2 : 1)))
scan_rows_kernel(Shape sh, Bufs bf, int tiles_per_wave, float* dst) {
    using v8 = typename Mfma<DT>::v8;
    constexpr int KS = D / 32;
    constexpr int X = 4 * NT;          // rows a lane owns: row 16 t + 4 j + i at x = 4 t + i
    const int G = sh.G, M = sh.M;
    // Workgroup -> (key stream bx of kv head kvh of cache sequence bc, row block blk).  With several
    // row blocks the blocks of one key stream take neighbouring slots of one XCD (workgroups go
    // to the XCDs round-robin by linear id), so they walk the same key tiles at the same time
    // and all but the first read of a tile are served by that XCD's L2.
    int bx = blockIdx.x, kvh = blockIdx.y, bc = (int)blockIdx.z / sh.n_qblk, blk = (int)blockIdx.z % sh.n_qblk;
    {
        const int gx = gridDim.x, gy = gridDim.y, streams = gx * gy * sh.Bc;
        if (sh.n_qblk > 1 && streams % 8 == 0) {
            const int lin = bx + gx * (kvh + gy * (int)blockIdx.z);
            const int slot = lin >> 3, stream = (slot / sh.n_qblk) * 8 + (lin & 7);
            blk = slot % sh.n_qblk;
            bx = stream % gx;
            kvh = (stream / gx) % gy;
            bc = stream / (gx * gy);
        }
    }
    // the M * G (query, head) rows of the KV head, query-major, are cut into blocks of 16 NT rows
    const int row0 = blk * 16 * NT;                                   // first row of the block
    const int R = M * G - row0 < 16 * NT ? M * G - row0 : 16 * NT;    // its rows
    const int lane = lane_id();
    const int j = lane >> 4, n = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t Nc = bf.len[bc];
    const int64_t N = prefix_len(Nc, sh.window);      // longest searched prefix of the sequence's queries

    // row rr of the block is head kvh * G + (row0 + rr) % G of query (row0 + rr) / G
    auto head_of = [&](int rr) -> int64_t {
        return ((int64_t)bc * M + (row0 + rr) / G) * sh.Hq + (int64_t)kvh * G + (row0 + rr) % G;
    };
    // candidates per score bin (tail_bin()) of each row, counted as they leave the stage
    __shared__ uint32_t hist_lds[MODE == MODE_FILTER ? 16 * NT * kTailBins : 1];
    if (MODE == MODE_FILTER) {
        for (int i = threadIdx.x; i < 16 * NT * kTailBins; i += kScanWaves * kWave) hist_lds[i] = 0;
        __syncthreads();
    }
    auto prefix_of = [&](int rr) -> int {   // keys row rr searches (0 for rows the block does not have)
        if (rr >= R) return 0;
        const int m = (row0 + rr) / G;
        return (int)prefix_len(Nc - (sh.causal ? M - 1 - m : 0), sh.window);
    };

    int64_t n_items = N;
    int stride = 1;
    if (MODE == MODE_SAMPLE) {
        if (N == 0) return;
        Plan pl = make_plan(N, sh.k < N ? sh.k : (int)N);
        n_items = pl.n_samp;
        stride = pl.stride;
    }
    const int64_t n_tiles_all = (n_items + 63) / 64;
    int64_t tile, tile_end, tile_step;
    if (MODE == MODE_FILTER) {
        tile = (int64_t)bx * kScanWaves + wave;
        tile_step = (int64_t)gridDim.x * kScanWaves;
        tile_end = n_tiles_all;
    } else {
        const int64_t tile0 = (int64_t)bx * tiles_per_wave * kScanWaves;
        if (tile0 >= n_tiles_all) return;
        tile = tile0 + wave;
        tile_step = kScanWaves;
        tile_end = tile0 + (int64_t)tiles_per_wave * kScanWaves;
        if (tile_end > n_tiles_all) tile_end = n_tiles_all;
    }

    // operand A of row tile t: lane (j, m) holds channels 32 s + 8 j .. +7 of row 16 t + m
    v8 qa[NT][KS];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int rr = 16 * t + n;
        const v8* p = reinterpret_cast<const v8*>(static_cast<const char*>(bf.q) + head_of(rr < R ? rr : 0) * (D * 2)) + j;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            v8 v = p[4 * s];
            if (rr >= R) v = v8{};
            qa[t][s] = v;
        }
    }
    const char* Kh = static_cast<const char*>(bf.K) + ((int64_t)bc * sh.Hkv + kvh) * sh.Ncap * (D * 2);

    // the rows this lane owns
    auto row_at = [&](int x) { return 16 * (x >> 2) + 4 * j + (x & 3); };
    int vh[X];              // head of each row (a 32-bit index: heads are few)
    int P[X];
    float thr[X], top[X];
    int nl[X], ng[X];       // staged / already appended candidates (uniform over the 16 lanes of the row)
#pragma unroll
    for (int x = 0; x < X; ++x) {
        int rr = row_at(x);
        asm volatile("" : "+v"(rr));     // the row's bins are read here, not kept in registers across the tile loop
        vh[x] = (int)head_of(rr < R ? rr : 0);
        P[x] = prefix_of(rr);
        thr[x] = (MODE == MODE_FILTER && rr < R) ? bf.thr[vh[x]] : INFINITY;
        top[x] = -INFINITY;
        nl[x] = 0;
        ng[x] = 0;
    }
    const int seg_cap = sh.seg_cap, n_seg = sh.n_seg;
    const int sid = bx * kScanWaves + wave;
    // tail_bin() parameters of each row, a copy per wave (read when the wave's staged candidates are counted)
    __shared__ float rows_all_lds[MODE == MODE_FILTER ? kScanWaves * 16 * NT * 2 : 1];
    float* const rows_lds = rows_all_lds + (MODE == MODE_FILTER ? wave * 16 * NT * 2 : 0);
    if (MODE == MODE_FILTER) {
#pragma unroll
        for (int x = 0; x < X; ++x) {
            const float2 lw = *reinterpret_cast<const float2*>(bf.bins + 2 * vh[x]);
            if (n == 0) *reinterpret_cast<float2*>(rows_lds + 2 * row_at(x)) = lw;
        }
    }
    __shared__ uint64_t stage_lds[MODE == MODE_FILTER ? kScanWaves * 16 * NT * kStageRow : 1];
    uint64_t* const st0 = stage_lds + (MODE == MODE_FILTER ? wave * 16 * NT * kStageRow : 0);

    // append the staged candidates of the rows at x (one per lane group) to their segments, up to
    // the last whole run of kCandChunk entries unless `final` (see stage_flush)
    auto flush = [&](int x, int& nl_i, int& ng_i, int64_t vh_i, bool final) {
        wave_sync();
        uint64_t* list = bf.cand + vh_i * (int64_t)sh.cand_cap;
        uint64_t* src = st0 + row_at(x) * kStageRow;
        const int total = ng_i + nl_i;
        const int f = (final ? total : (total & ~(kCandChunk - 1))) - ng_i;
        int rr = row_at(x);
        asm volatile("" : "+v"(rr));     // the row's bins are read here, not kept in registers across the tile loop
        const float bin_lo = rows_lds[2 * rr], bin_inv = rows_lds[2 * rr + 1];
        uint32_t* const hist = hist_lds + rr * kTailBins;
        for (int e = n; e < f; e += 16) {
            const int slot = ng_i + e;
            const uint64_t ent = src[e];
            if (slot < seg_cap) list[cand_slot(slot, sid, n_seg)] = ent;
            atomicAdd(&hist[tail_bin(__uint_as_float((uint32_t)(ent >> 32)), bin_lo, bin_inv)], 1u);   // also past a full segment
        }
        const int r = f > 0 ? nl_i - f : nl_i;          // < kCandChunk <= 16 after a flush
        const bool mv = f > 0 && n < r;
        const uint64_t keep = mv ? src[f + n] : 0;
        wave_sync();
        if (mv) src[n] = keep;
        wave_sync();
        if (f > 0) ng_i += f;
        nl_i = r;
    };

    auto row_of = [&](int64_t item0, int slot) -> int64_t {
        int64_t p = item0 + slot;
        if (MODE == MODE_SAMPLE) {
            if (p > n_items - 1) p = n_items - 1;
            p = sample_pos((int)p, stride);
        }
        return p < N ? p : N - 1;
    };
    // Filter step of a tile.  A lane counts its own passing keys of each row slot (at most 4,
    // one per sub-tile), the counts of four row slots share a register (a byte each: a row has
    // at most 64 passing keys per tile), and one inclusive scan over the 16 lanes of the row
    // group (four DPP row shifts) ranks all of them at once: no per-row ballots, no scalar
    // round trips.  Staged order within a row: by lane, then sub-tile (the selection does not
    // depend on it).  A lane that has nothing to store for a (row slot, sub-tile) writes to a
    // scratch slot of its own instead, so the stores need no branches.  WHOLE: the tile lies
    // inside every row's searched prefix.
    const int Pmin = prefix_of(0);      // rows of a block search prefixes that grow with the row
    __shared__ uint64_t dummy_lds[MODE == MODE_FILTER ? kScanWaves * kWave : 1];
    uint64_t* const dummy = dummy_lds + (MODE == MODE_FILTER ? threadIdx.x : 0);
    auto filter = [&](auto whole_tag, const f32x4 (&c)[NT][4], int64_t item0) {
        constexpr bool WHOLE = decltype(whole_tag)::value;
        const int item_n = (int)item0 + n;              // positions fit 31 bits
        bool ps[X][4];
        uint32_t pk[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) pk[t] = 0;
#pragma unroll
        for (int x = 0; x < X; ++x) {
            uint32_t cnt = 0;
            float mx = top[x];
            const int Px = WHOLE ? 0 : prefix_of(row_at(x));    // (worked out again for the few tiles at the end: a register less per row)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float sc = c[x >> 2][g][x & 3];
                const bool valid = WHOLE || item_n + 16 * g < Px;
                if (valid) mx = fmaxf(mx, sc);
                ps[x][g] = valid && sc >= thr[x];
                cnt += ps[x][g] ? 1u : 0u;
            }
            top[x] = mx;
            pk[x >> 2] |= cnt << (8 * (x & 3));
        }
        uint32_t anyp = pk[0];
#pragma unroll
        for (int t = 1; t < NT; ++t) anyp |= pk[t];
        if (!__ballot(anyp != 0u)) return;              // (uniform) nothing passes anywhere in the tile
        uint32_t incl[NT], tot[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            uint32_t v = pk[t];
            v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);   // row_shr:1
            v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);   // row_shr:2
            v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4
            v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);   // row_shr:8
            incl[t] = v;
            tot[t] = (uint32_t)__builtin_amdgcn_ds_bpermute((lane | 15) << 2, (int)v);      // the group's last lane
        }
        bool full = false;
#pragma unroll
        for (int x = 0; x < X; ++x) full |= nl[x] + (int)((tot[x >> 2] >> (8 * (x & 3))) & 0xFFu) > kStageRow;
        if (__builtin_expect(__ballot(full) != 0, 0)) {
#pragma unroll
            for (int x = 0; x < X; ++x)
                if (__ballot(nl[x] + (int)((tot[x >> 2] >> (8 * (x & 3))) & 0xFFu) > kStageRow))
                    flush(x, nl[x], ng[x], vh[x], false);
        }
#pragma unroll
        for (int x = 0; x < X; ++x) {
            // bytes of incl are >= those of pk: the packed subtraction has no borrows
            int off = nl[x] + (int)(((incl[x >> 2] - pk[x >> 2]) >> (8 * (x & 3))) & 0xFFu);
            uint64_t* row_st = st0 + row_at(x) * kStageRow;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint64_t* where = ps[x][g] ? row_st + off : dummy;
                *where = ((uint64_t)__float_as_uint(c[x >> 2][g][x & 3] + 0.0f) << 32) | (uint64_t)(uint32_t)(item_n + 16 * g);
                off += ps[x][g] ? 1 : 0;
            }
            nl[x] += (int)((tot[x >> 2] >> (8 * (x & 3))) & 0xFFu);
        }
    };
    auto consume = [&](const f32x4 (&c)[NT][4], int64_t item0) {
        if (MODE == MODE_SAMPLE) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int64_t item = item0 + 16 * g + n;
                if (item < n_items) {
                    const int64_t pos = sample_pos((int)item, stride);
#pragma unroll
                    for (int x = 0; x < X; ++x)   // a sample past the row's own prefix does not count
                        if (row_at(x) < R)
                            bf.samp[(int64_t)vh[x] * sh.samp_cap + item] = pos < P[x] ? c[x >> 2][g][x & 3] : -INFINITY;
                }
            }
        } else if (MODE == MODE_FULL) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int64_t item = item0 + 16 * g + n;
#pragma unroll
                for (int x = 0; x < X; ++x)
                    if (item < P[x]) dst[(int64_t)vh[x] * sh.Ncap + item] = c[x >> 2][g][x & 3];
            }
        } else {
            if (item0 + 64 <= Pmin) filter(std::true_type{}, c, item0);
            else filter(std::false_type{}, c, item0);
        }
    };
    auto mac = [&](const v8 (&b)[4][KS], f32x4 (&c)[NT][4]) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                c[t][g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s) c[t][g] = Mfma<DT>::mac(qa[t][s], b[g][s], c[t][g]);
            }
        }
    };

    struct TileB { v8 b[4][KS]; } ba, bb;
    auto load_rows = [&](TileB& t, int64_t ti) { tile_load<DT, D>(Kh, [&](int slot) { return row_of(ti * 64, slot); }, t.b); };
    auto use = [&](TileB& t, int64_t ti) {
        f32x4 c[NT][4];
        mac(t.b, c);
        consume(c, ti * 64);
    };
    if (MODE == MODE_SAMPLE) {
        walk_tiles<ScanPipelined<D>::value>(tile, tile_end, tile_step, ba, bb, load_rows, use);
    } else if (MODE == MODE_FILTER) {
        // one tile per row of n_seg tiles (seg_tile()): the rows made of whole tiles only first, then the
        // last one or two (tiles beyond the cache are skipped, the one its end cuts short is loaded row by row)
        const int n_seg = (int)tile_step;
        const int sid_w = (int)tile;                            // this wave's segment
        const int64_t n_whole = N / 64;
        const int64_t rows_whole = n_whole / n_seg, rows_all = (n_tiles_all + n_seg - 1) / n_seg;
        const uint32_t lane_off = (uint32_t)((n * D + j * 8) * 2);
        walk_tiles<ScanPipelined<D>::value>(0, rows_whole, 1, ba, bb,
            [&](TileB& t, int64_t i) { tile_load_full<DT, D>(Kh + seg_tile(i, sid_w, n_seg) * (64 * D * 2), lane_off, t.b); },
            [&](TileB& t, int64_t i) { use(t, seg_tile(i, sid_w, n_seg)); });
        for (int64_t i = rows_whole; i < rows_all; ++i) {
            const int64_t ti = seg_tile(i, sid_w, n_seg);
            if (ti < n_tiles_all) {
                load_rows(ba, ti);
                use(ba, ti);
            }
        }
    } else {
        const int64_t n_whole = N / 64;
        const uint32_t lane_off = (uint32_t)((n * D + j * 8) * 2);
        tile = walk_tiles<ScanPipelined<D>::value>(tile, tile_end < n_whole ? tile_end : n_whole, tile_step, ba, bb,
                          [&](TileB& t, int64_t ti) { tile_load_full<DT, D>(Kh + ti * (64 * D * 2), lane_off, t.b); }, use);
        for (; tile < tile_end; tile += tile_step) {
            load_rows(ba, tile);
            use(ba, tile);
        }
    }
    if (MODE == MODE_FILTER) {
#pragma unroll
        for (int i = 0; i < X; ++i) {
            flush(i, nl[i], ng[i], vh[i], true);
            for (int o = 8; o > 0; o >>= 1) top[i] = fmaxf(top[i], wave_xor(top[i], o));
            if (n == 0 && row_at(i) < R) {
                bf.seg_cnt[(int64_t)vh[i] * n_seg + sid] = (uint32_t)ng[i];
                bf.seg_max[(int64_t)vh[i] * n_seg + sid] = top[i];
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < R * kTailBins; i += kScanWaves * kWave)
            bf.hist[(head_of(i / kTailBins) * sh.hist_cap + bx) * kTailBins + i % kTailBins] = hist_lds[i];
    }
}

// Plain FMA scoring for what the MFMA kernels do not take (fp32 caches): a row of D elements is spread over D*e/16 lanes, 16 bytes each.
template <int DT>
__global__ void __launch_bounds__(256)
scan_generic_kernel(Shape sh, Bufs bf, int rows_per_block, float* dst) {
    constexpr int EPL = Elem<DT>::kPerLoad;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int G = sh.G, D = sh.D;
    const int64_t head0 = (int64_t)b * sh.Hq + (int64_t)kvh * G;
    const int64_t N = prefix_len(visible_len(sh, bf, b), sh.window);
    const int64_t row_begin = (int64_t)blockIdx.x * rows_per_block;
    if (row_begin >= N) return;

    __shared__ float q_lds[16 * 256];
    for (int i = threadIdx.x; i < G * D; i += blockDim.x) {
        const char* qp = static_cast<const char*>(bf.q) + (head0 * D + i) * Elem<DT>::kBytes;
        float v;
        if (DT == DT_F32) v = *reinterpret_cast<const float*>(qp);
        else if (DT == DT_F16) v = (float)*reinterpret_cast<const _Float16*>(qp);
        else v = __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(qp) << 16);
        q_lds[i] = v;
    }
    __syncthreads();

    const int lpr = D / EPL;              // lanes per row (power of two, <= 64)
    const int rows_per_pass = blockDim.x / lpr;
    const int slot = threadIdx.x / lpr, chunk = threadIdx.x % lpr;
    const char* Kh = static_cast<const char*>(bf.K) +
                     ((int64_t)cache_seq(sh, b) * sh.Hkv + kvh) * sh.Ncap * D * Elem<DT>::kBytes;
    int64_t row_end = row_begin + rows_per_block;
    if (row_end > N) row_end = N;
    for (int64_t base = row_begin; base < row_end; base += rows_per_pass) {
        const int64_t row = base + slot;
        const bool valid = row < row_end;
        const int64_t lrow = valid ? row : row_end - 1;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(Kh + (lrow * D + chunk * EPL) * Elem<DT>::kBytes);
        float kf[EPL];
        Elem<DT>::widen(raw, kf);
        for (int r = 0; r < G; ++r) {
            const float* qr = q_lds + r * D + chunk * EPL;
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc = fmaf(kf[e], qr[e], acc);
            for (int m = 1; m < lpr; m <<= 1) acc += wave_xor(acc, m);
            if (valid && chunk == 0) dst[(head0 + r) * sh.Ncap + row] = acc;
        }
    }
}

bool scan_mfma_supported(const Shape& s) {
    return (s.dtype == DT_F16 || s.dtype == DT_BF16) && (s.D == 32 || s.D == 64 || s.D == 128 || s.D == 256) && s.G >= 1;
}

template <int MODE>
static hipError_t launch_mfma(const Shape& s, const Bufs& b, int64_t n_items, float* dst, hipStream_t st) {
    const bool rows = scan_row_tiles(s);
    const int tpw = tiles_per_wave_for(n_items, scan_grid_z(s), s.Hkv);
    const int64_t tiles = (n_items + 63) / 64;
    const int64_t per_wg = (int64_t)tpw * kScanWaves;
    dim3 grid((unsigned)((tiles + per_wg - 1) / per_wg), (unsigned)s.Hkv, (unsigned)(scan_grid_z(s)));
    dim3 block(kScanWaves * kWave);
#define TKA_LAUNCH(DT_, D_)                                                                                 \
    do {                                                                                                    \
        if (rows && s.row_tiles == 2)                                                                       \
            hipLaunchKernelGGL((scan_rows_kernel<DT_, D_, MODE, 2>), grid, block, 0, st, s, b, tpw, dst);   \
        else if (rows)                                                                                      \
            hipLaunchKernelGGL((scan_rows_kernel<DT_, D_, MODE, 1>), grid, block, 0, st, s, b, tpw, dst);   \
        else hipLaunchKernelGGL((scan_mfma_kernel<DT_, D_, MODE>), grid, block, 0, st, s, b, tpw, dst);     \
    } while (0)
    if (s.dtype == DT_F16 && s.D == 128) TKA_LAUNCH(DT_F16, 128);
    else if (s.dtype == DT_F16 && s.D == 64) TKA_LAUNCH(DT_F16, 64);
    else if (s.dtype == DT_BF16 && s.D == 128) TKA_LAUNCH(DT_BF16, 128);
    else if (s.dtype == DT_BF16 && s.D == 64) TKA_LAUNCH(DT_BF16, 64);
    else if (s.dtype == DT_F16 && s.D == 256) TKA_LAUNCH(DT_F16, 256);
    else if (s.dtype == DT_BF16 && s.D == 256) TKA_LAUNCH(DT_BF16, 256);
    else if (s.dtype == DT_F16 && s.D == 32) TKA_LAUNCH(DT_F16, 32);
    else if (s.dtype == DT_BF16 && s.D == 32) TKA_LAUNCH(DT_BF16, 32);
    else return hipErrorInvalidValue;
#undef TKA_LAUNCH
    return hipGetLastError();
}

hipError_t launch_scan_sample(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st) {
    Plan pl = make_plan(Nmax, s.k);
    return launch_mfma<MODE_SAMPLE>(s, b, pl.n_samp, nullptr, st);
}

hipError_t launch_scan_filter_paged(const Shape& s, const Bufs& b, hipStream_t st) {
    if (scan_row_tiles(s)) return hipErrorInvalidValue;      // grouped scan only
    dim3 grid((unsigned)(s.n_seg / kScanWaves), (unsigned)s.Hkv, (unsigned)s.B);
    dim3 block(kScanWaves * kWave);
#define TKA_LAUNCH(DT_, D_) \
    hipLaunchKernelGGL((scan_mfma_kernel<DT_, D_, MODE_FILTER, true>), grid, block, 0, st, s, b, 0, (float*)nullptr)
    if (s.dtype == DT_F16 && s.D == 128) TKA_LAUNCH(DT_F16, 128);
    else if (s.dtype == DT_F16 && s.D == 64) TKA_LAUNCH(DT_F16, 64);
    else if (s.dtype == DT_BF16 && s.D == 128) TKA_LAUNCH(DT_BF16, 128);
    else if (s.dtype == DT_BF16 && s.D == 64) TKA_LAUNCH(DT_BF16, 64);
    else if (s.dtype == DT_F16 && s.D == 256) TKA_LAUNCH(DT_F16, 256);
    else if (s.dtype == DT_BF16 && s.D == 256) TKA_LAUNCH(DT_BF16, 256);
    else if (s.dtype == DT_F16 && s.D == 32) TKA_LAUNCH(DT_F16, 32);
    else if (s.dtype == DT_BF16 && s.D == 32) TKA_LAUNCH(DT_BF16, 32);
    else return hipErrorInvalidValue;
#undef TKA_LAUNCH
    return hipGetLastError();
}

hipError_t launch_scan_filter(const Shape& s, const Bufs& b, int64_t Nmax, hipStream_t st) {
    (void)Nmax;
    // one wave per candidate segment: n_seg / 4 workgroups per KV head
    const bool rows = scan_row_tiles(s);
    dim3 grid((unsigned)(s.n_seg / kScanWaves), (unsigned)s.Hkv, (unsigned)(scan_grid_z(s)));
    dim3 block(kScanWaves * kWave);
#define TKA_LAUNCH(DT_, D_)                                                                                  \
    do {                                                                                                     \
        if (rows && s.row_tiles == 2)                                                                        \
            hipLaunchKernelGGL((scan_rows_kernel<DT_, D_, MODE_FILTER, 2>), grid, block, 0, st, s, b, 0,     \
                               (float*)nullptr);                                                             \
        else if (rows)                                                                                       \
            hipLaunchKernelGGL((scan_rows_kernel<DT_, D_, MODE_FILTER, 1>), grid, block, 0, st, s, b, 0,     \
                               (float*)nullptr);                                                             \
        else                                                                                                 \
            hipLaunchKernelGGL((scan_mfma_kernel<DT_, D_, MODE_FILTER>), grid, block, 0, st, s, b, 0,        \
                               (float*)nullptr);                                                             \
    } while (0)
    if (s.dtype == DT_F16 && s.D == 128) TKA_LAUNCH(DT_F16, 128);
    else if (s.dtype == DT_F16 && s.D == 64) TKA_LAUNCH(DT_F16, 64);
    else if (s.dtype == DT_BF16 && s.D == 128) TKA_LAUNCH(DT_BF16, 128);
    else if (s.dtype == DT_BF16 && s.D == 64) TKA_LAUNCH(DT_BF16, 64);
    else if (s.dtype == DT_F16 && s.D == 256) TKA_LAUNCH(DT_F16, 256);
    else if (s.dtype == DT_BF16 && s.D == 256) TKA_LAUNCH(DT_BF16, 256);
    else if (s.dtype == DT_F16 && s.D == 32) TKA_LAUNCH(DT_F16, 32);
    else if (s.dtype == DT_BF16 && s.D == 32) TKA_LAUNCH(DT_BF16, 32);
    else return hipErrorInvalidValue;
#undef TKA_LAUNCH
    return hipGetLastError();
}

hipError_t launch_scan_full(const Shape& s, const Bufs& b, int64_t Nmax, float* dst, hipStream_t st) {
    if (scan_mfma_supported(s)) return launch_mfma<MODE_FULL>(s, b, Nmax, dst, st);
    const int epl = s.dtype == DT_F32 ? 4 : 8;
    const int lpr = s.D / epl;
    const int rows_per_pass = 256 / lpr;
    int64_t rows_per_block = (int64_t)rows_per_pass * 16;
    dim3 grid((unsigned)((Nmax + rows_per_block - 1) / rows_per_block), (unsigned)s.Hkv, (unsigned)s.B);
    if (s.dtype == DT_F32)
        hipLaunchKernelGGL((scan_generic_kernel<DT_F32>), grid, dim3(256), 0, st, s, b, (int)rows_per_block, dst);
    else if (s.dtype == DT_F16)
        hipLaunchKernelGGL((scan_generic_kernel<DT_F16>), grid, dim3(256), 0, st, s, b, (int)rows_per_block, dst);
    else
        hipLaunchKernelGGL((scan_generic_kernel<DT_BF16>), grid, dim3(256), 0, st, s, b, (int)rows_per_block, dst);
    return hipGetLastError();
}

}  // namespace tka
