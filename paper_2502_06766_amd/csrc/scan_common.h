// Pieces shared by the key scans (16-bit keys in scan.hip, int8 codes in index8.hip): the three
// uses of a scan, the per-(wave, head) candidate stage, and the grid shape of sample / full scans.
#pragma once
#include "device_utils.h"
#include "internal.h"

namespace tka {

enum { MODE_SAMPLE = 0, MODE_FILTER = 1, MODE_FULL = 2 };
constexpr int kScanWaves = 4;     // waves per scan workgroup

constexpr int kStage = 128;   // LDS staging slots per (wave, head)

// Candidates of one (wave, head): staged in LDS, appended to the wave's private segment
// of the head's global list in bursts.  Global stores in the tile loop would sit between
// the key loads in the wave's in-order memory queue and stall the prefetch.
struct CandStage {
    uint64_t* lds;      // kStage slots
    uint64_t* list;     // the head's candidate list (entry e of this wave at list[cand_slot(e, sid, n_seg)])
    int sid;            // this wave's segment
    int n_lds;          // staged entries (wave-uniform)
    int n_glob;         // entries already appended, may run past seg_cap (overflow is detected later)
};

// Appends the staged entries up to the last whole run of kCandChunk (all of them when
// `final`), so that every store but the last covers whole 128-byte lines; the remainder
// (fewer than kCandChunk entries) moves to the front of the stage.
__device__ __forceinline__ void stage_flush(CandStage& c, int seg_cap, int n_seg, bool final = false) {
    static_assert(kCandChunk <= kWave && kStage >= kWave + kCandChunk, "stage too small for an aligned flush");
    wave_sync();
    const int total = c.n_glob + c.n_lds;
    const int f = (final ? total : (total & ~(kCandChunk - 1))) - c.n_glob;     // entries to append now
    for (int i = lane_id(); i < f; i += kWave) {
        const int slot = c.n_glob + i;
        if (slot < seg_cap) c.list[cand_slot(slot, c.sid, n_seg)] = c.lds[i];
    }
    const int r = f > 0 ? c.n_lds - f : c.n_lds;
    if (f > 0) {
        const uint64_t keep = lane_id() < r ? c.lds[f + lane_id()] : 0;
        wave_sync();
        if (lane_id() < r) c.lds[lane_id()] = keep;
        c.n_glob += f;
    }
    wave_sync();
    c.n_lds = r;
}

// Keep the keys of one head whose score reaches the head's threshold.  `hist` (LDS, kTailBins
// counters of this head, or null) counts the kept keys per score bin.
__device__ __forceinline__ void filter_head(float score, float thr, CandStage& c, bool valid, int64_t item,
                                            int seg_cap, int n_seg, uint32_t* hist = nullptr, float bin_lo = 0.f, float bin_inv = 0.f) {
    const float sc = score + 0.0f;
    const bool pass = valid && sc >= thr;
    const uint64_t m = __ballot(pass);
    if (m) {
        const int add = __popcll(m);
        if (c.n_lds + add > kStage) stage_flush(c, seg_cap, n_seg);
        if (pass) {
            c.lds[c.n_lds + mask_rank(m)] = ((uint64_t)__float_as_uint(sc) << 32) | (uint64_t)(uint32_t)item;
            if (hist) atomicAdd(&hist[tail_bin(sc, bin_lo, bin_inv)], 1u);
        }
        c.n_lds += add;
    }
}

// Tile that wave segment `sid` takes in row i of the filter scan.  The tiles of a key stream form rows of
// n_seg consecutive tiles (n_seg a power of two), one tile per segment and row; each row is dealt to the
// segments rotated by a pseudo-random amount.  Consecutive tiles still go to consecutive segments, so a run
// of high scores spreads over neighbouring segments, and a pattern that repeats along the sequence (equally
// long documents with their hot tokens at the same place, say) does not put all its tiles into the same few
// segments, as the plain dealing sid, sid + n_seg, ... would.
__host__ __device__ inline int64_t seg_tile(int64_t i, int sid, int n_seg) {
    const uint32_t rot = ((uint32_t)i * 0x9E3779B1u) >> 12;
    return i * n_seg + (int64_t)(((uint32_t)sid + rot) & (uint32_t)(n_seg - 1));
}

inline int tiles_per_wave_for(int64_t n_items, int B, int Hkv) {
    // aim at ~16 workgroups per CU over the whole grid, at least 1 tile and at most 32 per wave
    const int64_t tiles = (n_items + 63) / 64;
    const int64_t want_wgs = 4096 / ((int64_t)B * Hkv > 0 ? (int64_t)B * Hkv : 1);
    int64_t tpw = tiles / (kScanWaves * (want_wgs > 0 ? want_wgs : 1));
    if (tpw < 1) tpw = 1;
    if (tpw > 64) tpw = 64;
    return (int)tpw;
}

}  // namespace tka
