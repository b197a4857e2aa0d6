// Layout of the opaque workspace inside distsim_events and the visiting order of simulate.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace distsim {

constexpr int kMaxPP = 64;
constexpr int kMaxM = 1 << 16;
constexpr int kClasses = 7;                 // lanes per candidate: 64, 32, 16, 8, 4, 2, 1
constexpr int kMBins = 1024;                // micro-batch count is clamped to this for ordering only
constexpr int kBinsPerClass = 2 * kMBins;   // schedule x m
constexpr int kBins = kClasses * kBinsPerClass;

// Header words kept in device memory (int64 each).
enum {
    H_CLASS_START = 0,             // [kClasses+1] first sorted position of each class
    H_ITEM_START = 8,              // [kClasses+1] first wave-item of each class
    H_NUM_ITEMS = 16,              // total wave-items
    H_WORDS = 32
};

struct Workspace {
    // layer-event prefix tables, entry [row*(L+1) + l] = sum over layers < l
    int64_t *pfc, *pbc, *pg;       // row = variant
    int64_t *pfa, *pba;            // row = variant*kMaxPP + (pp-1): in-stage communication incl. all-to-all
    int32_t *npp;                  // [C] stages owned (0 unless status OK)
    int32_t *key;                  // [C] ordering bin, -1 = not simulated
    int64_t *block_sums;           // [scan blocks]
    int32_t *bin_count;            // [kBins]
    int32_t *bin_start;            // [kBins+1]
    int32_t *bin_fill;             // [kBins]
    int64_t *hdr;                  // [H_WORDS]
    // candidates in visiting order
    int32_t *s_cand, *s_meta, *s_m, *s_dp;   // meta = pp | schedule << 8 | variant << 16 ; pp == 0: skip
    int64_t *s_off;
};

constexpr int kScanBlock = 256;
constexpr int kScanItems = 8;
constexpr int kScanChunk = kScanBlock * kScanItems;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Carves the workspace; returns the bytes used.  base may be null (size query).
inline size_t carve(Workspace& w, void* base, int32_t L, int32_t V, int64_t C) {
    size_t off = 0;
    char* b = (char*)base;
    auto take = [&](size_t bytes) { void* p = b ? (void*)(b + off) : nullptr; off += align256(bytes); return p; };
    const size_t row = (size_t)(L + 1) * sizeof(int64_t);
    const size_t Cc = (size_t)(C > 0 ? C : 1);
    w.pfc = (int64_t*)take(row * V);
    w.pbc = (int64_t*)take(row * V);
    w.pg = (int64_t*)take(row * V);
    w.pfa = (int64_t*)take(row * V * kMaxPP);
    w.pba = (int64_t*)take(row * V * kMaxPP);
    w.npp = (int32_t*)take(Cc * 4);
    w.key = (int32_t*)take(Cc * 4);
    w.block_sums = (int64_t*)take(((Cc + kScanChunk - 1) / kScanChunk + 1) * 8);
    w.bin_count = (int32_t*)take((size_t)kBins * 4);
    w.bin_start = (int32_t*)take((size_t)(kBins + 1) * 4);
    w.bin_fill = (int32_t*)take((size_t)kBins * 4);
    w.hdr = (int64_t*)take(H_WORDS * 8);
    w.s_cand = (int32_t*)take(Cc * 4);
    w.s_meta = (int32_t*)take(Cc * 4);
    w.s_m = (int32_t*)take(Cc * 4);
    w.s_dp = (int32_t*)take(Cc * 4);
    w.s_off = (int64_t*)take(Cc * 8);
    return off;
}

}  // namespace distsim
