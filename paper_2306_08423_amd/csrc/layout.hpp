// Layout of the opaque workspace inside distsim_events and the visiting order of simulate.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace distsim {

constexpr int kMaxPP = 64;
constexpr int kMaxM = 1 << 16;
constexpr int kMaxV = 16;                   // tensor-parallel variants of a cost table
constexpr int kMaxSlots = 2048;             // (virtual stage, micro-batch) pairs of an explicit schedule
// Compiled explicit schedules (k_compile_schedules): the first kSchedCap schedules, as far as their
// blocks lie in the first kSchedOpsCap words of the schedule array, get a program; a program's ring
// pool has at most kSchedMaxPool entries, the candidates of a wavefront share kSchedWavePool.
constexpr int kSchedCap = 4096;
constexpr int64_t kSchedOpsCap = 1 << 17;
constexpr int kSchedMaxPool = 256, kSchedWavePool = 256;
struct SchedHdr {
    int32_t state;                 // kSchedTable / kSchedCompiled / kSchedInvalid / kSchedStuck
    int32_t n_rounds, depth;       // rounds of the program, entries per ring
    int32_t n_send;                // tasks that are followed by a transfer
};
constexpr int kClasses = 7;                 // lanes per candidate: 64, 32, 16, 8, 4, 2, 1
constexpr int kMBins = 1024;                // micro-batch count is clamped to this for ordering only
constexpr int kBinsPerClass = 2 * kMBins;   // schedule x m
// The second half of a class's bins (schedules other than GPipe), longest lists first in each part:
// the level sweeps' schedules by m (pairs of m share a bin above 512), then the interleaved
// candidates by m * chunks / 16, then those with an explicit schedule by m / 16 -- so that the
// kernels of the last two find their candidates side by side.
constexpr int kSubVirtual = 768, kSubExplicit = 896;
constexpr int kBins = kClasses * kBinsPerClass;
constexpr int kCombWords = 6;               // int64 words per entry of Workspace::comb

// Header words kept in device memory (int64 each).
enum {
    H_CLASS_START = 0,             // [kClasses+1] first sorted position of each class
    H_ITEM_START = 8,              // [kClasses+1] first wave-item of each class
    H_NUM_ITEMS = 16,              // total wave-items
    H_GPIPE_ITEMS = 17,            // [kClasses] leading wave-items of each class that hold only GPipe candidates
                                   //            (an even number; zero for the class of one lane per candidate)
    H_PAIRS = 24,                  // [2] pairs of wave-items that k_simulate / k_simulate_gpipe take (entries of Workspace::order)
    H_SCHED_TABLE = 26,            // explicit schedules without a compiled program (k_simulate_explicit takes their candidates)
    H_WORDS = 32
};

// One candidate in visiting order (32 bytes; the first 16 are all that simulate needs).
struct alignas(16) Desc {
    int32_t cand;                  // index in the caller's arrays
    int32_t meta;                  // pp | schedule << 8 | variant << 16 ; pp == 0: skip
    int32_t m, dp;
    int64_t poff;                  // offset of the partition in part_pool, -1 = uniform
    int64_t spare;                 // tensor-parallel size | chunks per device << 32
};

struct Workspace {
    // layer-event prefix tables, entry [row*(L+1) + l] = sum over layers < l
    int64_t *pfc, *pbc, *pg;       // row = variant
    int64_t *pfa, *pba;            // row = variant*kMaxPP + (pp-1): in-stage communication incl. all-to-all
    int64_t *p2p;                  // [(variant*L + l)*2 + link class]: p2p event of the activation after layer l
    // The same sums arranged for simulate, row = variant*kMaxPP + (pp-1), six words per entry l:
    //   pfc+pfa, pbc+pba | pfc+pbc, pg | p2p event (intra-, inter-node) of the activation that
    //   enters layer l
    // so that a stage's composed events come from two neighbouring-in-memory places.  No activation
    // enters layer 0: the last two words of a row's first entry hold the row's mask of inter-node
    // stage boundaries (bit s: positions s and s + 1 start on different nodes) and, as a double, the
    // reciprocal of dp * beta of the gradient all-reduce over the row's dp group.
    int64_t *comb;
    int32_t *key;                  // [C] ordering bin | variant << 24, -1 = not simulated
    int32_t *bin_count;            // [kBins]
    int32_t *bin_start;            // [kBins+1]
    int32_t *rank;                 // [C] position of the candidate inside its bin
    int64_t *hdr;                  // [H_WORDS]
    int32_t *vtp;                  // [kMaxV] the cost table's variant -> tensor-parallel size (a copy: the calls
                                   //         after event generation do not see the cost table any more)
    Desc *desc;                    // [C] candidates in visiting order
    // Order in which the sweep kernels take pairs of wave-items, longest sweeps first (k_pair_order):
    // entry = index of the pair's first wave-item | 1 << 31 when the next item belongs to the pair too;
    // order[0]: k_simulate's pairs, order[1]: k_simulate_gpipe's.
    int32_t *order[2];             // [order_cap] each
    int64_t order_cap;
    int64_t *sched_ops;            // [kSchedOpsCap + 8] programs of the explicit schedules, word for word beside schedule_words
    SchedHdr *sched_hdr;           // [kSchedCap]
};

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
    w.p2p = (int64_t*)take((size_t)V * L * 2 * sizeof(int64_t));
    w.comb = (int64_t*)take(row * V * kMaxPP * kCombWords);
    w.key = (int32_t*)take(Cc * 4);
    w.bin_count = (int32_t*)take((size_t)kBins * 4);
    w.bin_start = (int32_t*)take((size_t)(kBins + 1) * 4);
    w.rank = (int32_t*)take(Cc * 4);
    w.hdr = (int64_t*)take(H_WORDS * 8);
    w.vtp = (int32_t*)take(kMaxV * 4);
    w.desc = (Desc*)take(Cc * sizeof(Desc));
    w.order_cap = (int64_t)(Cc / 2 + kClasses + 1);       // a class of n items has (n + 1) / 2 pairs
    w.order[0] = (int32_t*)take((size_t)w.order_cap * 4);
    w.order[1] = (int32_t*)take((size_t)w.order_cap * 4);
    w.sched_ops = (int64_t*)take((size_t)(kSchedOpsCap + 8) * 8);
    w.sched_hdr = (SchedHdr*)take((size_t)kSchedCap * sizeof(SchedHdr));
    return off;
}

}  // namespace distsim
