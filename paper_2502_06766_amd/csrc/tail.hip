// Tail of the filtered path: exact top-k among the candidates the key scan kept, softmax
// over the k selected scores and weighted sum of their value rows (the knn_search result
// and the attention step of Algorithm 1 of arXiv 2502.06766), in two kernels that use the
// whole chip instead of one workgroup per head.
//
// The scan leaves, beside every head's candidate list, the number of candidates each of
// its workgroups found per score bin (64 bins above the head's threshold, monotone in the
// score).  From these counts every workgroup of the first kernel derives, on its own and
// without any exchange, the bin B the k-th largest score falls in: candidates in higher
// bins are selected for certain, candidates in lower bins are not, and only those of bin B
// (a few hundred) still have to be ranked exactly.
//
//   tail_gather_kernel  many workgroups per head, each over the candidates of a few scan
//                       workgroups: writes the certain winners to idx / vals at offsets known
//                       from the counts, copies bin B's candidates to the head's boundary
//                       list, and accumulates the softmax-weighted value rows of its winners
//                       (weights relative to the head's largest score, which the scan reported;
//                       the rows are asked for as soon as the winners are known, before it is
//                       known where they go in idx / vals).
//   tail_finish_kernel  one workgroup per head: the missing winners among the boundary list (ranked
//                       by direct comparison of composite keys, lower position wins ties; a
//                       crowded list is first sorted into sub-bins over its own score range, a
//                       list of mostly tied scores goes through the radix select), their value
//                       rows, the sum of all partials in a fixed order, normalisation, padding
//                       of idx / vals.
//
// A head whose candidate list is unusable (a segment overflowed, the sampled threshold came
// out above the k-th score, or its sequence cannot be filtered at all) is redone exactly
// inside the same two launches (modes RESCAN and DENSE below): the workgroups of the first
// kernel score the keys of their scan workgroups again with the MFMA tile routine of the scan,
// and either sort them from the k-th score's bin up (known from the scan's counts) into the
// head's segments and go on as with a list, or write all scores to the score buffer, over
// which the second kernel selects densely.  Nothing is launched for the common case.
#include "device_utils.h"
#include "gather_common.h"
#include "internal.h"
#include "scan_common.h"
#include "scan_tiles.h"
#include "select_common.h"

namespace tka {

enum { TAIL_NORMAL = 0, TAIL_REDO = 1, TAIL_EMPTY = 2 };
struct TailRec { uint32_t state, above, need, have; };   // what tail_finish_kernel needs to know of a head

constexpr int kTailThreads = 256;
constexpr int kTailWaves = kTailThreads / kWave;
constexpr int kTailStage = 128;      // winners a wave stages before it fetches their value rows
static_assert(kTailWaves == kScanWaves && kTailBins == kWave, "wave w of a tail workgroup takes the segments of wave w of the scan");

// How a head's selection is obtained (uniform over the workgroups of the head):
//   LIST    from its candidate list (the usual case);
//   RESCAN  the list is unusable (a segment overflowed) but the scan's per-bin counts, which go on where
//           the list stops, cover at least k keys: every workgroup scores the keys of its scan
//           workgroups again, keeps those from the k-th score's bin up in the segments the scan
//           would have put them in, and sorts them as it would have sorted list entries;
//   DENSE   neither (fewer than k keys reached the threshold, or too many share the k-th score's bin):
//           all scores go to the score buffer and the second kernel selects over the full row.
enum { MODE_LIST = 0, MODE_RESCAN = 1, MODE_DENSE = 2 };

struct HeadSel {          // what a workgroup needs to sort a head's candidates (uniform over the workgroup)
    int mode, binB;
    uint32_t above, have, emit_at, bnd_at;   // certain winners, bin-B candidates; this workgroup's first output slots
    float hmax;
};

struct TailShared {
    uint32_t red[3][kTailWaves];
    uint32_t part[2][kTailWaves][kTailBins];
    uint32_t sel[6];
    uint32_t cnt[kTailWaves][2];
    int32_t st_pos[kTailWaves][kTailStage];
    float st_w[kTailWaves][kTailStage];
};

// What the scan left for head bh: candidates in all segments, longest segment, largest score
// key any scanning wave saw.  All threads of the workgroup call it and get the same values.
__device__ __forceinline__ void seg_summary(const Shape& sh, const Bufs& bf, int64_t bh, TailShared& sm,
                                            uint32_t& total, uint32_t& max_len, uint32_t& kmx) {
    uint32_t sum = 0, mxl = 0, km = 0;
    for (int g = threadIdx.x; g < sh.n_seg; g += kTailThreads) {
        const uint32_t c = bf.seg_cnt[bh * sh.n_seg + g];
        const uint32_t m = score_key(bf.seg_max[bh * sh.n_seg + g]);
        sum += c;
        mxl = c > mxl ? c : mxl;
        km = m > km ? m : km;
    }
    for (int o = 32; o > 0; o >>= 1) {
        sum += __shfl_xor(sum, o, kWave);
        const uint32_t t = __shfl_xor(mxl, o, kWave), u = __shfl_xor(km, o, kWave);
        mxl = t > mxl ? t : mxl;
        km = u > km ? u : km;
    }
    if (lane_id() == 0) {
        const int w = threadIdx.x >> 6;
        sm.red[0][w] = sum; sm.red[1][w] = mxl; sm.red[2][w] = km;
    }
    __syncthreads();
    total = 0; max_len = 0; kmx = 0;
#pragma unroll
    for (int w = 0; w < kTailWaves; ++w) {
        total += sm.red[0][w];
        max_len = sm.red[1][w] > max_len ? sm.red[1][w] : max_len;
        kmx = sm.red[2][w] > kmx ? sm.red[2][w] : kmx;
    }
}

// Everything a workgroup whose first scan workgroup is j0 needs to know of head bh.  `h_all` / `h_before`
// are this thread's share of the head's per-bin candidate counts (bin tid % 64, a quarter of the scan
// workgroups; all of them, and those before j0).  All threads call it once and get the same result.
__device__ __forceinline__ HeadSel analyse_head(const Shape& sh, const Bufs& bf, int64_t bh, int k_eff, uint32_t h_all,
                                                uint32_t h_before, TailShared& sm) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    sm.part[0][wave][threadIdx.x & (kTailBins - 1)] = h_all;
    sm.part[1][wave][threadIdx.x & (kTailBins - 1)] = h_before;
    if (threadIdx.x == 0) sm.sel[5] = 0u;
    uint32_t total, max_len, kmx;
    seg_summary(sh, bf, bh, sm, total, max_len, kmx);      // (its barrier also covers the stores above)
    if (wave == 0) {
        // lane l looks at bin kTailBins - 1 - l: prefix sums run from the highest bin down
        const int bin = kTailBins - 1 - lane;
        uint32_t all = 0, before = 0;
#pragma unroll
        for (int p = 0; p < kTailWaves; ++p) { all += sm.part[0][p][bin]; before += sm.part[1][p][bin]; }
        uint32_t ia = all, ib = before;
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t va = __shfl_up(ia, o, kWave), vb = __shfl_up(ib, o, kWave);
            if (lane >= o) { ia += va; ib += vb; }
        }
        const uint32_t run = ia - all;
        if (run < (uint32_t)k_eff && (uint32_t)k_eff <= ia) {        // at most one lane
            sm.sel[0] = (uint32_t)bin;           // B: the bin the k-th score falls in
            sm.sel[1] = run;                     // candidates in higher bins: selected for certain
            sm.sel[2] = all;                     // candidates in bin B
            sm.sel[3] = ib - before;             // certain winners of the scan workgroups before j0
            sm.sel[4] = before;                  // bin-B candidates of the scan workgroups before j0
            sm.sel[5] = 1u;                      // the counts cover k_eff keys
        }
    }
    __syncthreads();
    HeadSel hs;
    hs.binB = (int)sm.sel[0]; hs.above = sm.sel[1]; hs.have = sm.sel[2]; hs.emit_at = sm.sel[3]; hs.bnd_at = sm.sel[4];
    const bool counted = sm.sel[5] != 0u;
    hs.hmax = key_score(kmx);
    // the bin of the k-th score has to fit the boundary list, and the keys sorted again their list
    const bool bnd_ok = counted && hs.have <= (uint32_t)sh.bnd_cap;
    const bool list_ok = !(bf.flags[bh] & 4u) && max_len <= (uint32_t)sh.seg_cap && total >= (uint32_t)k_eff && bnd_ok;
    hs.mode = list_ok ? MODE_LIST
                      : (bnd_ok && !sh.no_rescan && (uint64_t)hs.above + hs.have <= (uint64_t)sh.cand_cap ? MODE_RESCAN : MODE_DENSE);
    return hs;
}

template <int DT, int D, bool WIN>
__global__ void __launch_bounds__(kTailThreads) tail_gather_kernel(Shape sh, Bufs bf, float scale_log2e) {
    using v8 = typename Mfma<DT>::v8;
    if (WIN && (int)blockIdx.x >= sh.tail_wgs) {
        // the recent-token window rides in the same launch: the workgroups behind the head's tail_wgs leave the
        // partial sums of its chunks in the slots behind theirs (they wait for nothing of the search)
        static_assert(kTailThreads == 256, "window_chunk() is written for workgroups of 256 threads");
        __shared__ GatherShared win_sm;
        const int chunk = (int)blockIdx.x - sh.tail_wgs;
        window_chunk<DT>(sh, bf, scale_log2e, chunk, blockIdx.y, blockIdx.z, sh.tail_wgs + chunk, win_sm);
        return;
    }
    constexpr int EPL = 8;                 // elements per 16-byte load
    constexpr int LPR = D / EPL;           // lanes per value row
    constexpr int RPW = kWave / LPR;       // rows a wave fetches per load instruction
    constexpr int U = 4;                   // independent rows in flight per lane group
    constexpr int R = 2;                   // batches of 64 candidates a wave keeps in registers between its two passes
    __shared__ TailShared sm;
    __shared__ float s_acc[kTailWaves][D + 1];

    const int awg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t bh = (int64_t)b * sh.Hq + h;
    TailRec* rec = reinterpret_cast<TailRec*>(bf.tailrec) + bh;

    // Everything the prologue needs from memory is asked for before anything is waited for: this
    // kernel is a chain of dependent steps per workgroup, and every load it waits for on its own
    // costs a full trip to memory (what the scan wrote is in no cache of this compute unit).
    const int n_wg = sh.n_seg / kScanWaves;                          // scan workgroups that fed this head
    const int j0 = awg * sh.tail_spw;
    const int j1 = j0 + sh.tail_spw < n_wg ? j0 + sh.tail_spw : n_wg;
    const float bin_lo = bf.bins[2 * bh], bin_inv = bf.bins[2 * bh + 1];
    uint64_t* const list = bf.cand + bh * (int64_t)sh.cand_cap;
    uint32_t h_all = 0, h_before = 0;
    {
        const uint32_t* hp = bf.hist + bh * (int64_t)sh.hist_cap * kTailBins;
        const int bin = tid & (kTailBins - 1), part = tid >> 6;      // kTailBins == kWave: one wave per part
#pragma unroll 8
        for (int j = part; j < n_wg; j += kTailWaves) {
            const uint32_t c = hp[j * kTailBins + bin];
            h_all += c;
            h_before += j < j0 ? c : 0u;
        }
    }
    // the first candidates of this wave's first segment, before their number is known (any slot of
    // the list may be read; what lies beyond the segment's length is ignored below)
    uint64_t saved[R];
    {
        const int g_first = j0 * kScanWaves + wave;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t slot = cand_slot(r * kWave + lane, g_first, sh.n_seg);
            saved[r] = list[slot < sh.cand_cap ? slot : 0];
        }
    }
    const int64_t N = prefix_len(visible_len(sh, bf, b), sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    if (k_eff == 0) {                      // nothing to search for this sequence
        if (awg == 0 && tid == 0) *rec = TailRec{TAIL_EMPTY, 0u, 0u, 0u};
        return;
    }
    const HeadSel hs = analyse_head(sh, bf, bh, k_eff, h_all, h_before, sm);
    if (awg == 0 && tid == 0) {
        const bool dense = hs.mode == MODE_DENSE;
        rec->state = dense ? (uint32_t)TAIL_REDO : (uint32_t)TAIL_NORMAL;
        rec->above = dense ? 0u : hs.above;
        rec->need = dense ? 0u : (uint32_t)k_eff - hs.above;
        rec->have = dense ? 0u : hs.have;
        bf.hmax[bh] = hs.hmax;
        if (hs.mode != MODE_LIST && !(bf.flags[bh] & 5u)) atomicAdd(bf.fallback_total, 1u);   // a list that should have been usable
    }

    const uint32_t* scnt = bf.seg_cnt + bh * sh.n_seg;
    if (hs.mode != MODE_LIST) {
        // ---- The list is unusable: the keys of my scan workgroups' tiles are scored again with the scan's
        // own arithmetic, 16 keys at a time (a quarter of the scan's tile keeps this rarely used branch from
        // setting the register budget of the kernel): lane (jj, n) loads the chunks 4 s + jj of key n, and
        // every group of four accumulator rows holds the score of key n in its first row.
        // Every score goes to the score buffer.  RESCAN: keys from bin B up also go to the head's candidate
        // list again, into the segment the scan would have put them in; the segments' new lengths are kept
        // apart from the scan's (other workgroups may still be judging the head by those).
        // Operand A holds this head alone (rows 0, 4, 8, 12; the others zero), so that accumulator element 0 is
        // its score in every lane: no choice among the four elements by the head's place in its group between
        // the MFMAs and the read of their result.  (A wave-uniform choice compiles to a branch there, and the
        // read behind that branch came too early after the last MFMA: the scores of a group's first head were
        // those of half-finished accumulators.)
        v8 qa[D / 32];
        load_query_a<DT, D>(bf.q, bh, 1, qa);
        const char* Kh = static_cast<const char*>(bf.K) + ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * (D * 2);
        const int jj = lane >> 4, n = lane & 15;
        const bool rescan = hs.mode == MODE_RESCAN;
        const int64_t n_tiles = (N + 63) / 64;
        for (int j = j0; j < j1; ++j) {
            const int sid = j * kScanWaves + wave;
            uint32_t cnt = 0;                                           // entries written to segment sid (uniform over the wave)
            for (int64_t row = 0; row * sh.n_seg < n_tiles; ++row) {    // the tiles the scan dealt to segment sid
                const int64_t tile = seg_tile(row, sid, sh.n_seg);
                if (tile >= n_tiles) continue;
#pragma unroll
                for (int sub = 0; sub < 4; ++sub) {
                    const int64_t key = tile * 64 + sub * 16 + n;
                    const v8* p = reinterpret_cast<const v8*>(Kh + (key < N ? key : N - 1) * (D * 2)) + jj;
                    v8 kb[D / 32];
#pragma unroll
                    for (int s = 0; s < D / 32; ++s) kb[s] = p[4 * s];
                    f32x4 acc4 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < D / 32; ++s) acc4 = Mfma<DT>::mac(qa[s], kb[s], acc4);
                    const float sc = acc4[0] + 0.0f;
                    const bool mine = jj == 0 && key < N;               // every lane group holds the same scores: the first one writes
                    if (mine) bf.scores[bh * sh.Ncap + key] = sc;        // (also when sorting again: should a segment overflow once more, the second kernel selects over this row)
                    const bool keep = mine && rescan && tail_bin(sc, bin_lo, bin_inv) >= hs.binB;
                    const uint64_t m = __ballot(keep);
                    if (keep) {
                        const uint32_t e = cnt + (uint32_t)mask_rank(m);
                        if (e < (uint32_t)sh.seg_cap)
                            list[cand_slot(e, sid, sh.n_seg)] = ((uint64_t)__float_as_uint(sc) << 32) | (uint64_t)(uint32_t)key;
                    }
                    cnt += (uint32_t)__popcll(m);
                }
            }
            if (lane == 0 && rescan) {
                bf.seg_cnt2[bh * sh.n_seg + sid] = cnt < (uint32_t)sh.seg_cap ? cnt : (uint32_t)sh.seg_cap;
                if (cnt > (uint32_t)sh.seg_cap) atomicOr(&bf.flags[bh], 2u);           // does not fit: the second kernel selects densely
            }
        }
        if (!rescan) return;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();                      // the segments written above are read below by other lanes; a line of the
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // old list may sit in this compute unit's cache (it was read early on)
        scnt = bf.seg_cnt2 + bh * sh.n_seg;
        saved[0] = saved[1] = 0ull;           // (not carried through this branch: nothing is cached for a list written again)
    }
    const bool cached = hs.mode == MODE_LIST;     // the first R batches of this wave's first segment are in saved[]

    // ---- first pass over my candidates: how many certain winners / bin-B candidates each wave has, and the
    // winners' positions and softmax weights into the wave's LDS stage (their value rows can be fetched
    // before it is known where they go in idx / vals).  Wave w takes segment 4 j + w of every scan workgroup
    // j of mine, 64 candidates at a time; the first R batches stay in registers for the second pass.
    const char* Vh = static_cast<const char*>(bf.V) +
                     ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * (D * 2);
    const int rs = lane / LPR, c = lane % LPR;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float lsum = 0.f;
    int n_st = 0;                                                    // staged winners (uniform over the wave)
    const uint32_t n_last = (uint32_t)(N - 1);                       // (N >= 1 here, and below 2^31)
    // one round of staged rows: U per lane group, asked for by ask_round() and added up by add_round()
    auto ask_round = [&](int r0, float (&w)[U], u32x4 (&raw)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * RPW + rs;
            const bool ok = r < n_st;
            const uint32_t p32 = (uint32_t)sm.st_pos[wave][ok ? r : 0];
            const int64_t pos = (int64_t)(p32 < n_last ? p32 : n_last);   // (entries are positions below N; never read beyond the cache)
            w[u] = ok ? sm.st_w[wave][r] : 0.f;
            raw[u] = *reinterpret_cast<const u32x4*>(Vh + (pos * D + c * EPL) * 2);
        }
    };
    auto add_round = [&](const float (&w)[U], const u32x4 (&raw)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[EPL];
            Elem<DT>::widen(raw[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(w[u], vf[e], acc[e]);
            lsum += w[u];
        }
    };
    auto fetch_staged = [&](int r_first) {                           // rows r_first .. n_st - 1 of the stage
        for (int r0 = r_first; r0 < n_st; r0 += RPW * U) {
            float w[U];
            u32x4 raw[U];
            ask_round(r0, w, raw);
            add_round(w, raw);
        }
    };
    uint32_t nw = 0, nb = 0;                                         // (uniform over the wave)
    {
        int bi = 0;
        for (int j = j0; j < j1; ++j) {
            const int g = j * kScanWaves + wave;
            const uint32_t cnt = scnt[g];
            for (uint32_t e0 = 0; e0 < cnt; e0 += kWave, ++bi) {
                const uint32_t e = e0 + lane;
                const bool valid = e < cnt;
                uint64_t ent;
                if (cached && j == j0 && bi < R) ent = bi == 0 ? saved[0] : saved[1];
                else {
                    ent = list[cand_slot(valid ? e : 0, g, sh.n_seg)];
                    if (bi < R) { if (bi == 0) saved[0] = ent; else saved[1] = ent; }
                }
                const float sc = __uint_as_float((uint32_t)(ent >> 32));
                const int bin = tail_bin(sc, bin_lo, bin_inv);
                const bool win = valid && bin > hs.binB;
                const uint64_t mw = __ballot(win), me = __ballot(valid && bin == hs.binB);
                if (n_st > kTailStage - kWave) {                     // the stage is full: its rows are fetched now
                    wave_sync();
                    fetch_staged(0);
                    wave_sync();
                    n_st = 0;
                }
                if (win) {
                    const int r = n_st + mask_rank(mw);
                    sm.st_pos[wave][r] = (int32_t)(uint32_t)ent;
                    sm.st_w[wave][r] = exp2f((sc - hs.hmax) * scale_log2e);
                }
                const int addw = __popcll(mw);
                n_st += addw;
                nw += (uint32_t)addw;
                nb += (uint32_t)__popcll(me);
            }
        }
    }
    static_assert(R == 2, "the register cache of candidate batches is written out for two batches");
    // the first round of value rows is asked for now: it is under way while the waves exchange their counts and
    // the second pass writes the selection
    wave_sync();
    float w_first[U];
    u32x4 raw_first[U];
    if (n_st > 0) ask_round(0, w_first, raw_first);                  // (uniform over the wave)
    if (lane == 0) { sm.cnt[wave][0] = nw; sm.cnt[wave][1] = nb; }
    __syncthreads();
    uint32_t emit_at = hs.emit_at, bnd_at = hs.bnd_at;
    for (int w = 0; w < wave; ++w) { emit_at += sm.cnt[w][0]; bnd_at += sm.cnt[w][1]; }

    // ---- second pass: write winners and boundary candidates where the counts put them
    int32_t* idx = bf.sel_idx + bh * sh.k;
    float* vals = bf.sel_val + bh * sh.k;
    uint64_t* bnd = bf.bnd + bh * (int64_t)sh.bnd_cap;
    {
        int bi = 0;
        for (int j = j0; j < j1; ++j) {
            const int g = j * kScanWaves + wave;
            const uint32_t cnt = scnt[g];
            for (uint32_t e0 = 0; e0 < cnt; e0 += kWave, ++bi) {
                const uint32_t e = e0 + lane;
                const bool valid = e < cnt;
                uint64_t ent;
                if (bi < R) ent = bi == 0 ? saved[0] : saved[1];
                else ent = list[cand_slot(valid ? e : 0, g, sh.n_seg)];
                const float sc = __uint_as_float((uint32_t)(ent >> 32));
                const int bin = tail_bin(sc, bin_lo, bin_inv);
                const bool win = valid && bin > hs.binB, edge = valid && bin == hs.binB;
                const uint64_t mw = __ballot(win), me = __ballot(edge);
                if (win) {
                    const uint32_t o = emit_at + (uint32_t)mask_rank(mw);
                    if (o < (uint32_t)k_eff) {            // always true for a consistent list; guards the output buffers
                        idx[o] = (int32_t)(uint32_t)ent;
                        vals[o] = sc;
                    }
                }
                if (edge) {
                    const uint32_t o = bnd_at + (uint32_t)mask_rank(me);
                    if (o < (uint32_t)sh.bnd_cap) bnd[o] = ent;
                }
                emit_at += (uint32_t)__popcll(mw);
                bnd_at += (uint32_t)__popcll(me);
            }
        }
    }
    if (n_st > 0) add_round(w_first, raw_first);
    fetch_staged(RPW * U);

    // ---- this workgroup's partial sum (weights relative to the head's largest score)
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += wave_xor(acc[e], o);
        lsum += wave_xor(lsum, o);
    }
    if (rs == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[wave][c * EPL + e] = acc[e];
        if (c == 0) s_acc[wave][D] = lsum;
    }
    __syncthreads();
    float* pacc = bf.part_acc + (bh * sh.n_chunk_cap + awg) * D;
    for (int t = tid; t < D; t += kTailThreads) pacc[t] = (s_acc[0][t] + s_acc[1][t]) + (s_acc[2][t] + s_acc[3][t]);
    if (tid == 0) {
        bf.part_l[bh * sh.n_chunk_cap + awg] = (s_acc[0][D] + s_acc[1][D]) + (s_acc[2][D] + s_acc[3][D]);
        bf.part_m[bh * sh.n_chunk_cap + awg] = hs.hmax;
    }
}

// Candidates of the boundary bin: a dense list of (score bits << 32 | position) entries.
template <int NT>
struct SrcListT {
    static constexpr int kThreads = NT;
    const uint64_t* ent;
    int64_t n;
    uint32_t* pos_lds;       // LDS: inverted positions of the cached slots, [slot j][thread]
    typedef uint64_t raw_t;
    __device__ __forceinline__ int64_t slots() const { return n; }
    __device__ __forceinline__ bool valid(int64_t i) const { return i < n; }
    __device__ __forceinline__ const uint64_t* where(int64_t i) const { return ent + i; }
    __device__ __forceinline__ uint32_t key(uint64_t e) const { return score_key(__uint_as_float((uint32_t)(e >> 32))); }
    __device__ __forceinline__ uint32_t ipos(uint64_t e, int64_t) const { return 0xFFFFFFFFu - (uint32_t)e; }
    __device__ __forceinline__ void stash(int j, uint64_t e) const { pos_lds[j * NT + (int)threadIdx.x] = 0xFFFFFFFFu - (uint32_t)e; }
    __device__ __forceinline__ uint32_t cached_ipos(int j) const { return pos_lds[j * NT + (int)threadIdx.x]; }
};

constexpr int kFinishInner = 2048;     // candidates the finishing workgroup ranks by direct comparison at most
constexpr int kFinishSmall = 4096;     // boundary candidates the finishing workgroup holds in registers; more go through the radix select

// Rank of each of this thread's CI items among the composite keys in LDS (number of keys that
// beat it), by comparing with every key: all lanes read the same key at a time (an LDS
// broadcast), eight reads in flight.  `n8` is the list length rounded up to a multiple of eight,
// the padding holds keys that beat nothing.
template <int CI>
__device__ __forceinline__ void rank_by_comparison(const uint64_t* keys, int n8, const uint64_t (&mine)[CI], uint32_t (&rank)[CI]) {
#pragma unroll
    for (int i = 0; i < CI; ++i) rank[i] = 0;
    for (int base = 0; base < n8; base += 8) {
        uint64_t o[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) o[u] = keys[base + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int i = 0; i < CI; ++i) rank[i] += o[u] > mine[i] ? 1u : 0u;
        }
    }
}

template <int DT, int NT>
__global__ void __launch_bounds__(NT) tail_finish_kernel(Shape sh, Bufs bf, float scale, float scale_log2e) {
    constexpr int EPL = 8, NW = NT / kWave, CPT = 4, U = 8;       // U: value rows in flight per lane group
    constexpr int CIMAX = kFinishSmall / NT;       // boundary candidates per thread on the small path
    __shared__ SelShared sm;
    __shared__ uint32_t pos_lds[CPT * NT];
    __shared__ __align__(16) uint64_t s_keys[kFinishInner + 8];
    __shared__ int32_t s_pos[kFinishSmall];
    __shared__ float s_w[kFinishSmall];
    __shared__ float s_acc[NW][256 + 1];
    __shared__ float s_red[NT];
    __shared__ uint32_t s_cnt[2][NW];
    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int64_t bh = (int64_t)b * sh.Hq + h;
    const int D = sh.D;
    const int64_t N = prefix_len(visible_len(sh, bf, b), sh.window);
    const int k_eff = sh.k < N ? sh.k : (int)N;
    TailRec rec = reinterpret_cast<const TailRec*>(bf.tailrec)[bh];
    if (bf.flags[bh] & 2u) rec.state = TAIL_REDO;     // the keys sorted again did not fit their segments
    float hmax = bf.hmax[bh];                 // the first kernel's, unless the head is redone
    // the first boundary candidates are asked for before their number is known (any slot of the
    // list may be read; what lies beyond `have` is ignored below)
    uint64_t ent[CIMAX];
#pragma unroll
    for (int i = 0; i < CIMAX; ++i) ent[i] = (i * NT + tid < sh.bnd_cap) ? bf.bnd[bh * (int64_t)sh.bnd_cap + i * NT + tid] : 0ull;
    int32_t* idx = bf.sel_idx + bh * sh.k;
    float* vals = bf.sel_val + bh * sh.k;
    // With a recent-token window (always attended, outside the search) the window's partial sums, each
    // relative to its own largest score, sit in the slots behind the first kernel's: one softmax over both
    // parts by the usual rescaling.  `at`, `lt`: this thread's output element and the weight total of the
    // retrieved part relative to `m_top` (lt == 0: nothing retrieved).
    const int n_win = (sh.window + kGatherRows - 1) / kGatherRows;
    auto write_out = [&](float at, float lt, float m_top) {
        const int e = tid % D;
        float M = lt > 0.f ? m_top : -INFINITY;
        const float* pl = bf.part_l + bh * sh.n_chunk_cap + sh.tail_wgs;
        const float* pm = bf.part_m + bh * sh.n_chunk_cap + sh.tail_wgs;
        const float* pa = bf.part_acc + (bh * sh.n_chunk_cap + sh.tail_wgs) * (int64_t)D + e;
        for (int s = 0; s < n_win; ++s)
            if (pl[s] > 0.f) M = fmaxf(M, pm[s]);
        if (n_win > 0 && M > -INFINITY) {
            const float f0 = lt > 0.f ? exp2f((m_top - M) * scale_log2e) : 0.f;
            at *= f0; lt *= f0;
            for (int s = 0; s < n_win; ++s) {
                const float ls = pl[s];
                if (ls > 0.f) {
                    const float f = exp2f((pm[s] - M) * scale_log2e);
                    lt = fmaf(ls, f, lt);
                    at = fmaf(pa[(int64_t)s * D], f, at);
                }
            }
        }
        const bool any = lt > 0.f;
        bf.out[bh * D + e] = any ? at / lt : 0.f;
        if (tid == 0 && bf.lse) bf.lse[bh] = any ? M * scale + logf(lt) : -INFINITY;
    };
    if (rec.state == TAIL_EMPTY || k_eff == 0) {      // nothing to search for this sequence
        pad_outputs(0, sh.k, idx, vals);
        if (tid == 0) bf.hmax[bh] = -INFINITY;
        if (tid < D) write_out(0.f, 0.f, -INFINITY);
        return;
    }
    // the partial sums of the first kernel's workgroups, NT / D threads per output element (asked for
    // first: nothing below depends on them until the end)
    const int n_parts = rec.state == TAIL_NORMAL ? sh.tail_wgs : 0;
    const int parts = NT / D, e_out = tid % D, part = tid / D;
    constexpr int PV = 32;                    // partials per thread whose loads stay in flight until the end
    float pv[PV], a_parts = 0.f, l_parts = 0.f;
    {
        const float* pa = bf.part_acc + bh * sh.n_chunk_cap * (int64_t)D + e_out;
#pragma unroll
        for (int u = 0; u < PV; ++u) {
            const int s = part + u * parts;
            pv[u] = s < n_parts ? pa[(int64_t)s * D] : 0.f;
        }
        for (int s0 = part + PV * parts; s0 < n_parts; s0 += 8 * parts) {      // (more than PV * parts partials: eight loads at a time, added in the same order)
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int s = s0 + u * parts;
                t[u] = s < n_parts ? pa[(int64_t)s * D] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) a_parts += t[u];
        }
        for (int s = tid; s < n_parts; s += NT) l_parts += bf.part_l[bh * sh.n_chunk_cap + s];
    }
    const int lpr = D / EPL, rpw = kWave / lpr;
    const int rs = lane / lpr, c = lane % lpr;
    const char* Vh = static_cast<const char*>(bf.V) + ((int64_t)cache_seq(sh, b) * sh.Hkv + h / sh.G) * sh.Ncap * D * 2;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float lsum = 0.f;
    const uint32_t n_last = (uint32_t)(N > 0 ? N - 1 : 0);
    // weighted value rows j0 .. j1 of a list of (position, weight) pairs
    auto gather_rows = [&](int j0, int j1, auto pos_of, auto weight_of) {
        const int step = NW * rpw;
        for (int j = j0 + wave * rpw + rs; j < j1; j += U * step) {
            int64_t r[U];
            float w[U];
            u32x4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = j + u * step;
                const bool ok = jj < j1;
                const uint32_t p32 = (uint32_t)pos_of(ok ? jj : j);
                r[u] = (int64_t)(p32 < n_last ? p32 : n_last);       // (never read beyond the cache, whatever an entry holds)
                w[u] = ok ? weight_of(jj) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) raw[u] = *reinterpret_cast<const u32x4*>(Vh + (r[u] * D + c * EPL) * 2);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[EPL];
                Elem<DT>::widen(raw[u], vf);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(w[u], vf[e], acc[e]);
                lsum += w[u];
            }
        }
    };

    // How the winners among the boundary candidates are found (uniform over the workgroup).
    enum { BY_REDO, BY_RADIX, BY_SUBBINS, BY_RANKING };
    const int have = (int)rec.have, need = (int)rec.need;
    int how = rec.state == TAIL_REDO ? BY_REDO : have > kFinishSmall ? BY_RADIX : have > NT ? BY_SUBBINS : BY_RANKING;
    int sb[CIMAX], sbin = 0, sure = 0, m = 0;
    if (how == BY_SUBBINS) {
        // Many boundary candidates (scores that come in clusters put a whole cluster into the bin of the
        // k-th score): sort them once more into kBins sub-bins over their own score range, take the
        // sub-bins above the one the need-th best falls in as they are, and rank only that one.
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int i = 0; i < CIMAX; ++i) {
            const float sc = __uint_as_float((uint32_t)(ent[i] >> 32));
            if (i * NT + tid < have) { lo = fminf(lo, sc); hi = fmaxf(hi, sc); }
        }
        for (int o = 32; o > 0; o >>= 1) { lo = fminf(lo, wave_xor(lo, o)); hi = fmaxf(hi, wave_xor(hi, o)); }
        if (lane == 0) { s_red[wave] = lo; s_red[NW + wave] = hi; }
        for (int i = tid; i < kBins; i += NT) sm.hist[i] = 0;
        if (tid == 0) { sm.bin = 0u; sm.above = 0u; sm.cb = (uint32_t)have; }     // (overwritten below: 1 <= need <= have)
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) { lo = fminf(lo, s_red[w]); hi = fmaxf(hi, s_red[NW + w]); }
        const float sub_inv = hi > lo ? (float)(kBins - 1) / (hi - lo) : 0.f;
#pragma unroll
        for (int i = 0; i < CIMAX; ++i) {
            const float sc = __uint_as_float((uint32_t)(ent[i] >> 32));
            sb[i] = i * NT + tid < have ? (int)fminf((sc - lo) * sub_inv, (float)(kBins - 1)) : -1;   // monotone in the score
            if (sb[i] >= 0) atomicAdd(&sm.hist[sb[i]], 1u);
        }
        __syncthreads();
        {   // the sub-bin in which the counts, summed from the top, reach `need`: thread t looks at the two bins 2t, 2t+1 from the top
            static_assert(kBins == 2 * NT, "two sub-bins per thread");
            const uint32_t c0 = sm.hist[kBins - 1 - 2 * tid], c1 = sm.hist[kBins - 2 - 2 * tid];
            uint32_t inc = c0 + c1;
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t v = __shfl_up(inc, o, kWave);
                if (lane >= o) inc += v;
            }
            if (lane == kWave - 1) s_cnt[0][wave] = inc;
            __syncthreads();
            uint32_t before = inc - (c0 + c1);
            for (int w = 0; w < wave; ++w) before += s_cnt[0][w];
            if (before < (uint32_t)need && (uint32_t)need <= before + c0) { sm.bin = (uint32_t)(kBins - 1 - 2 * tid); sm.above = before; sm.cb = c0; }
            else if (before + c0 < (uint32_t)need && (uint32_t)need <= before + c0 + c1) {
                sm.bin = (uint32_t)(kBins - 2 - 2 * tid); sm.above = before + c0; sm.cb = c1;
            }
            __syncthreads();
        }
        sbin = (int)sm.bin; sure = (int)sm.above; m = (int)sm.cb;
        if (m > kFinishInner) how = BY_RADIX;      // (nearly) all of them tie: the radix select breaks ties by position
    }
    if (how == BY_REDO) {
        // every score of the head is in the score buffer: exact selection over the full row
        hmax = key_score(wg_select_dense<NT, 8>(sh, bf, bh, N, k_eff, sm));     // writes idx, vals, padding, hmax
        __syncthreads();                      // idx / vals written above are read below
        gather_rows(0, k_eff, [&](int j) { return (int64_t)idx[j]; },
                    [&](int j) { return exp2f((vals[j] - hmax) * scale_log2e); });
    } else if (how == BY_RADIX) {
        // a boundary bin this full (massive ties, or a sample that misjudged the k-th score): radix select
        const SrcListT<NT> src{bf.bnd + bh * (int64_t)sh.bnd_cap, (int64_t)rec.have, pos_lds};
        const Items<CPT, SrcListT<NT>> items(src);
        wg_topk_emit(items, (int)rec.need, sh.k - (int)rec.above, idx + rec.above, vals + rec.above, sm);
        __syncthreads();
        gather_rows((int)rec.above, k_eff, [&](int j) { return (int64_t)idx[j]; },
                    [&](int j) { return exp2f((vals[j] - hmax) * scale_log2e); });
    } else {
        if (how == BY_SUBBINS) {
            // fixed order (wave, slot, lane) for both the certain winners and the entries still to rank
            uint32_t tot_w = 0, tot_e = 0;
#pragma unroll
            for (int i = 0; i < CIMAX; ++i) {
                tot_w += (uint32_t)__popcll(__ballot(sb[i] > sbin));
                tot_e += (uint32_t)__popcll(__ballot(sb[i] == sbin));
            }
            if (lane == 0) { s_cnt[0][wave] = tot_w; s_cnt[1][wave] = tot_e; }
            __syncthreads();
            uint32_t run_w = 0, run_e = 0;
            for (int w = 0; w < wave; ++w) { run_w += s_cnt[0][w]; run_e += s_cnt[1][w]; }
#pragma unroll
            for (int i = 0; i < CIMAX; ++i) {
                const bool win = sb[i] > sbin, edge = sb[i] == sbin;
                const uint64_t mw = __ballot(win), me = __ballot(edge);
                const float sc = __uint_as_float((uint32_t)(ent[i] >> 32));
                if (win) {
                    const uint32_t o = run_w + (uint32_t)mask_rank(mw);
                    if (o < (uint32_t)need) {         // always true; guards the buffers
                        idx[rec.above + o] = (int32_t)(uint32_t)ent[i];
                        vals[rec.above + o] = sc;
                        s_pos[o] = (int32_t)(uint32_t)ent[i];
                        s_w[o] = exp2f((sc - hmax) * scale_log2e);
                    }
                }
                if (edge) {
                    const uint32_t o = run_e + (uint32_t)mask_rank(me);
                    if (o < (uint32_t)kFinishInner) s_keys[o] = ((uint64_t)score_key(sc) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)ent[i]);
                }
                run_w += (uint32_t)__popcll(mw);
                run_e += (uint32_t)__popcll(me);
            }
            const int m8 = (m + 7) & ~7;
            if (tid < m8 - m) s_keys[m + tid] = 0ull;                     // padding: beats nothing
            __syncthreads();
            const uint32_t need2 = (uint32_t)(need - sure);               // 1 .. m of the ranked entries win
            for (int j = tid; j < m; j += NT) {
                const uint64_t m1[1] = {s_keys[j]};
                uint32_t r1[1];
                rank_by_comparison<1>(s_keys, m8, m1, r1);
                if (r1[0] < need2) {
                    const uint32_t o = (uint32_t)sure + r1[0];
                    const float sc = key_score((uint32_t)(m1[0] >> 32));
                    const int32_t pos = (int32_t)(0xFFFFFFFFu - (uint32_t)m1[0]);
                    idx[rec.above + o] = pos;
                    vals[rec.above + o] = sc;
                    s_pos[o] = pos;
                    s_w[o] = exp2f((sc - hmax) * scale_log2e);
                }
            }
        } else {
            // The usual case, at most one boundary candidate per thread: each is ranked against all others
            // by its composite key (score key, then inverted position: larger beats smaller, equal scores go
            // to the lower position, no two keys are equal), and the `need` best are the missing winners.
            const uint64_t mine[1] = {tid < have ? ((uint64_t)score_key(__uint_as_float((uint32_t)(ent[0] >> 32))) << 32) |
                                                       (uint64_t)(0xFFFFFFFFu - (uint32_t)ent[0])
                                                 : ~0ull};                    // nothing beats an empty slot's key
            if (tid < have) s_keys[tid] = mine[0];
            const int have8 = (have + 7) & ~7;
            if (tid < have8 - have) s_keys[have + tid] = 0ull;               // padding: beats nothing
            __syncthreads();
            uint32_t rank[1];
            rank_by_comparison<1>(s_keys, have8, mine, rank);
            // winners in thread order
            const bool win = tid < have && rank[0] < (uint32_t)need;
            const uint64_t mw = __ballot(win);
            if (lane == 0) sm.wave_tot[wave] = (uint32_t)__popcll(mw);
            __syncthreads();
            uint32_t run = 0;
            for (int w = 0; w < wave; ++w) run += sm.wave_tot[w];
            if (win) {
                const uint32_t o = run + (uint32_t)mask_rank(mw);
                if (o < (uint32_t)need) {         // always true; guards the buffers
                    const float sc = __uint_as_float((uint32_t)(ent[0] >> 32));
                    idx[rec.above + o] = (int32_t)(uint32_t)ent[0];
                    vals[rec.above + o] = sc;
                    s_pos[o] = (int32_t)(uint32_t)ent[0];
                    s_w[o] = exp2f((sc - hmax) * scale_log2e);
                }
            }
        }
        pad_outputs(k_eff, sh.k, idx, vals);
        __syncthreads();
        gather_rows(0, need, [&](int j) { return (int64_t)s_pos[j]; }, [&](int j) { return s_w[j]; });
    }

    for (int o = lpr; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += wave_xor(acc[e], o);
        lsum += wave_xor(lsum, o);
    }
    __syncthreads();                          // sm.wave_tot is reused below
    if (rs == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_acc[wave][c * EPL + e] = acc[e];
        if (c == 0) s_acc[wave][256] = lsum;
    }
    for (int o = 32; o > 0; o >>= 1) l_parts += wave_xor(l_parts, o);          // fixed tree: same result every run
#pragma unroll
    for (int u = 0; u < PV; ++u) a_parts += pv[u];                             // fixed order
    s_red[tid] = a_parts;
    if (lane == 0) sm.wave_tot[wave] = __float_as_uint(l_parts);
    __syncthreads();
    if (tid < D) {
        float lt = 0.f, at = 0.f;
        for (int w = 0; w < NW; ++w) lt += __uint_as_float(sm.wave_tot[w]) + s_acc[w][256];
        for (int w = 0; w < NW; ++w) at += s_acc[w][e_out];
        for (int p = 0; p < parts; ++p) at += s_red[p * D + e_out];
        write_out(at, lt, hmax);
    }
}

bool tail_supported(const Shape& s) {
    const int n_win = (s.window + kGatherRows - 1) / kGatherRows;     // the window's partial sums follow the tail's
    return (!s.indexed || s.no_rescan) && (s.dtype == DT_F16 || s.dtype == DT_BF16) &&
           s.n_seg % kScanWaves == 0 && s.n_seg / kScanWaves <= s.hist_cap && s.tail_wgs + n_win <= s.n_chunk_cap;
}

hipError_t launch_tail(const Shape& s, const Bufs& b, hipStream_t st) {
    const float scale = 1.0f / sqrtf((float)s.D);
    const float scale_log2e = scale * 1.4426950408889634f;
    const int n_win = (s.window + kGatherRows - 1) / kGatherRows;     // chunks of the recent-token window, if any
    const dim3 grid_a((unsigned)(s.tail_wgs + n_win), (unsigned)s.Hq, (unsigned)s.B);
#define TKA_TAIL_A(DT_, D_)                                                                                              \
    do {                                                                                                                 \
        if (n_win) hipLaunchKernelGGL((tail_gather_kernel<DT_, D_, true>), grid_a, dim3(kTailThreads), 0, st, s, b, scale_log2e); \
        else hipLaunchKernelGGL((tail_gather_kernel<DT_, D_, false>), grid_a, dim3(kTailThreads), 0, st, s, b, scale_log2e);      \
    } while (0)
    if (s.dtype == DT_F16 && s.D == 128) TKA_TAIL_A(DT_F16, 128);
    else if (s.dtype == DT_BF16 && s.D == 128) TKA_TAIL_A(DT_BF16, 128);
    else if (s.dtype == DT_F16 && s.D == 64) TKA_TAIL_A(DT_F16, 64);
    else if (s.dtype == DT_BF16 && s.D == 64) TKA_TAIL_A(DT_BF16, 64);
    else if (s.dtype == DT_F16 && s.D == 256) TKA_TAIL_A(DT_F16, 256);
    else if (s.dtype == DT_BF16 && s.D == 256) TKA_TAIL_A(DT_BF16, 256);
    else if (s.dtype == DT_F16 && s.D == 32) TKA_TAIL_A(DT_F16, 32);
    else if (s.dtype == DT_BF16 && s.D == 32) TKA_TAIL_A(DT_BF16, 32);
    else return hipErrorInvalidValue;
#undef TKA_TAIL_A
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid_b((unsigned)s.Hq, (unsigned)s.B);
    if (s.dtype == DT_F16) hipLaunchKernelGGL((tail_finish_kernel<DT_F16, 256>), grid_b, dim3(256), 0, st, s, b, scale, scale_log2e);
    else hipLaunchKernelGGL((tail_finish_kernel<DT_BF16, 256>), grid_b, dim3(256), 0, st, s, b, scale, scale_log2e);
    return hipGetLastError();
}

}  // namespace tka
