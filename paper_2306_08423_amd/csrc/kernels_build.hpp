// Event-flow generation kernels: layer-event tables, candidate decoding, visiting order,
// per-stage composed events (Sec. 4.1 events -> Sec. 4.3 composed events).
#pragma once
#include "device_utils.hpp"
#include "layout.hpp"

namespace distsim {

struct CostsDev {
    int32_t L, V;
    const int32_t* variant_tp;
    const int64_t *fc, *bc, *fa, *ba, *act, *grad, *a2a;   // a2a may be null
};

struct CandDev {
    const int32_t *dp, *tp, *pp, *m;
    const uint8_t* schedule;
    const int64_t* part_off;
    const uint8_t* part_pool;
    int64_t part_pool_len;
    const int32_t* chunks;         // model chunks per device (interleaved schedule) / index of the explicit schedule; may be null
    int64_t n_schedules;           // explicit schedules
    const int64_t* schedule_off;   // [n_schedules + 1]
    const int32_t* schedule_words;
    int64_t schedule_words_len;
};

struct EventsDev {
    int64_t stage_cap;
    int32_t* status;
    int64_t* stage_pos;
    int64_t* stage_tab;
    int32_t* stage_layers;
    int64_t* num_events;
};

// One wave-item = 64 lanes = (64 >> sh) consecutive candidates of one class, 1 << sh lanes each.
// Item w owns the 64 entries [64 w, 64 w + 64) of every per-stage array.
struct Item {
    int sh;
    int64_t pos0, class_end;
};

// Candidates of the interleaved schedule keep their place in the visiting order (their per-stage
// rows are per device) but are simulated by k_simulate_virtual; the other sweeps see them as empty.
__device__ __forceinline__ bool is_interleaved(const Desc& d) { return ((d.meta >> 8) & 0xff) == 3; }
// ... and the explicit schedules (k_simulate_explicit); either kind is skipped by the level sweeps.
__device__ __forceinline__ bool is_explicit(const Desc& d) { return ((d.meta >> 8) & 0xff) == 4; }
__device__ __forceinline__ bool has_own_kernel(const Desc& d) { return ((d.meta >> 8) & 0xff) >= 3; }
// Positions in visiting order of class k's interleaved candidates / of those with an explicit schedule.
__device__ __forceinline__ void interleaved_range(const Workspace& ws, int k, int64_t& lo, int64_t& hi) {
    lo = ws.bin_start[k * kBinsPerClass + kMBins + kSubVirtual];
    hi = ws.bin_start[k * kBinsPerClass + kMBins + kSubExplicit];
}
__device__ __forceinline__ void explicit_range(const Workspace& ws, int k, int64_t& lo, int64_t& hi) {
    lo = ws.bin_start[k * kBinsPerClass + kMBins + kSubExplicit];
    hi = ws.bin_start[(k + 1) * kBinsPerClass];
}

__device__ __forceinline__ Item decode_item(const int64_t* __restrict__ hdr, int64_t w) {
    int k = 0;
#pragma unroll
    for (int i = 1; i < kClasses; i++) k += (w >= hdr[H_ITEM_START + i]) ? 1 : 0;
    Item it;
    it.sh = 6 - k;
    it.pos0 = hdr[H_CLASS_START + k] + ((w - hdr[H_ITEM_START + k]) << k);
    it.class_end = hdr[H_CLASS_START + k + 1];
    return it;
}

// ---------------------------------------------------------------------------------------
// Layer-event tables.  One wavefront per row.  Rows [0, V*kMaxPP): (variant, pp) -> prefix
// sums over layers of the in-stage communication events of a forward / backward pass: the
// layer's all-reduce event when tp > 1 (model-parallel mapping, Sec. 4.3) plus the all-to-all
// over the dp = N / (tp pp) group.  Rows with pp == 1 also produce the variant's computation
// and gradient-byte prefixes.  Event times are shared by all candidates that generate the
// same event (Sec. 3.2); so are the two possible p2p events (intra- / inter-node) of the
// activation that leaves each layer.
__global__ __launch_bounds__(64) void k_layer_tables(CostsDev co, ClusterDev cl, Workspace ws) {
    const int row = blockIdx.x;
    const int v = row / kMaxPP, pp = row % kMaxPP + 1;
    const int lane = threadIdx.x;
    if (row == 0 && lane == 0) ws.hdr[H_SCHED_TABLE] = 0;             // counted up by k_compile_schedules, which follows
    const int L = co.L;
    const int tp = co.variant_tp[v];
    int64_t dp = 1;
    if (tp >= 1 && (int64_t)tp * pp <= cl.num_devices && cl.num_devices % ((int64_t)tp * pp) == 0)
        dp = cl.num_devices / ((int64_t)tp * pp);
    int64_t* pfa = ws.pfa + (size_t)row * (L + 1);
    int64_t* pba = ws.pba + (size_t)row * (L + 1);
    const bool base = pp == 1;
    int64_t* pfc = ws.pfc + (size_t)v * (L + 1);
    int64_t* pbc = ws.pbc + (size_t)v * (L + 1);
    int64_t* pg = ws.pg + (size_t)v * (L + 1);
    int64_t* comb = ws.comb + (size_t)row * (L + 1) * kCombWords;
    int64_t c_fa = 0, c_ba = 0, c_fc = 0, c_bc = 0, c_g = 0;
    if (row == 0 && lane < co.V) ws.vtp[lane] = co.variant_tp[lane];
    if (lane == 0) {
        pfa[0] = 0; pba[0] = 0;
        if (base) { pfc[0] = 0; pbc[0] = 0; pg[0] = 0; }
        for (int k = 0; k < 4; k++) comb[k] = 0;
        // what an all-reduce over this row's dp group divides by, as a reciprocal (word 5 of the row's
        // first entry; word 4 follows below): dp * beta of the group's link class
        const double den = (double)dp * (double)cl.beta[dp <= cl.gpus_per_node ? 0 : 1];
        comb[5] = __double_as_longlong(1.0 / den);
    }
    {
        // Link classes of this row's stage boundaries (word 4 of the row's first entry): bit s is set
        // when the ranks of pipeline positions s and s + 1 start on different nodes.  Ranks are
        // ordered tp fastest, then dp, then pp, so position s starts at rank s * (N / pp); a position
        // of at least a node's worth of ranks starts on a node of its own.
        bool inter = false;
        if (cl.num_devices % pp == 0 && lane + 1 < pp) {
            const int64_t span = cl.num_devices / pp, g = cl.gpus_per_node;
            const int64_t a = span >= g ? lane : (lane * span) / g, b = span >= g ? lane + 1 : ((lane + 1) * span) / g;
            inter = a != b;
        }
        const uint64_t mask = __builtin_amdgcn_ballot_w64(inter);
        if (lane == 0) comb[4] = (int64_t)mask;
    }
    for (int l0 = 0; l0 < L; l0 += kWave) {
        const int l = l0 + lane;
        const bool in = l < L;
        const size_t i = (size_t)v * L + (in ? l : 0);
        int64_t x = 0;
        if (in && co.a2a) x = alltoall_ns(cl, dp, co.a2a[i]);
        int64_t f = in ? x + (tp > 1 ? co.fa[i] : 0) : 0;
        int64_t b = in ? x + (tp > 1 ? co.ba[i] : 0) : 0;
        f = wave_inclusive_sum(f) + c_fa;
        b = wave_inclusive_sum(b) + c_ba;
        const int64_t a = wave_inclusive_sum(in ? co.fc[i] : 0) + c_fc;
        const int64_t bb = wave_inclusive_sum(in ? co.bc[i] : 0) + c_bc;
        const int64_t g = wave_inclusive_sum(in ? co.grad[i] : 0) + c_g;
        if (in) {
            const int64_t p_intra = p2p_ns(cl, co.act[i], 0), p_inter = p2p_ns(cl, co.act[i], 1);
            pfa[l + 1] = f; pba[l + 1] = b;
            int64_t* e = comb + (size_t)(l + 1) * kCombWords;
            e[0] = a + f; e[1] = bb + b; e[2] = a + bb; e[3] = g; e[4] = p_intra; e[5] = p_inter;
            if (base) {
                pfc[l + 1] = a; pbc[l + 1] = bb; pg[l + 1] = g;
                ws.p2p[i * 2 + 0] = p_intra;
                ws.p2p[i * 2 + 1] = p_inter;
            }
        }
        c_fa = __shfl(f, kWave - 1, kWave);
        c_ba = __shfl(b, kWave - 1, kWave);
        c_fc = __shfl(a, kWave - 1, kWave);
        c_bc = __shfl(bb, kWave - 1, kWave);
        c_g = __shfl(g, kWave - 1, kWave);
    }
}

__global__ void k_clear_bins(Workspace ws) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < kBins) ws.bin_count[i] = 0;
}

// ---------------------------------------------------------------------------------------
// Candidate decoding.  Checks what can be checked in O(1) -- sizes, device count, table variant,
// schedule, partition offset -- and files the candidate into its ordering bin; the partition
// itself and the 2^53 range guard are checked per stage later.
// A workgroup takes kDecodeChunk consecutive candidates and counts them in a histogram in LDS;
// only the non-empty bins go to the global counters (one atomic each), which hands the
// workgroup its base rank in every bin.  rank[c] is the candidate's position inside its bin.
constexpr int kDecodeBlock = 1024;
constexpr int kDecodePer = 4;                 // candidates per thread
constexpr int kDecodeChunk = kDecodeBlock * kDecodePer;

__global__ __launch_bounds__(kDecodeBlock) void k_decode(CostsDev co, ClusterDev cl, CandDev ca, int64_t C,
                                                         Workspace ws, EventsDev ev) {
    __shared__ int32_t hist[kBins];
    for (int b = threadIdx.x; b < kBins; b += kDecodeBlock) hist[b] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kDecodeChunk + threadIdx.x;
    int key[kDecodePer], rank[kDecodePer];
#pragma unroll
    for (int j = 0; j < kDecodePer; j++) {
        const int64_t c = base + (int64_t)j * kDecodeBlock;
        key[j] = -1; rank[j] = 0;
        if (c >= C) continue;
        const int32_t dp = ca.dp[c], tp = ca.tp[c], pp = ca.pp[c], m = ca.m[c];
        const int sched = ca.schedule[c];
        const int64_t poff = ca.part_off[c];
        // ok: a strategy as far as O(1) checks can tell; sup: within what the kernels of this library take
        bool ok = dp >= 1 && tp >= 1 && pp >= 1 && m >= 1 && sched <= 4 && pp <= co.L && pp <= kMaxPP;
        bool sup = m <= kMaxM;
        ok = ok && (int64_t)dp * tp * pp == (int64_t)cl.num_devices;
        int64_t parts = pp;                      // parts of the layer partition
        int64_t slots3 = 0;                      // interleaved: slots per direction of a device's list
        if (ok && sched == 3) {                  // interleaved: pp * chunks virtual stages
            const int64_t vch = ca.chunks ? ca.chunks[c] : 0;      // no chunk counts: invalid
            slots3 = (int64_t)m * vch;
            parts = (int64_t)pp * vch;
            ok = vch >= 1 && parts <= co.L && m % pp == 0;
            sup = sup && parts <= kMaxPP;
        }
        if (ok && sched == 4) {                  // explicit: the head of its schedule block; the kernel checks the rest
            const int64_t id = ca.chunks ? ca.chunks[c] : -1;
            ok = id >= 0 && id < ca.n_schedules && ca.schedule_off && ca.schedule_words;
            if (ok) {
                const int64_t o = ca.schedule_off[id], n = ca.schedule_off[id + 1] - o;
                ok = o >= 0 && n >= 5 + pp + 1 && o <= ca.schedule_words_len && n <= ca.schedule_words_len - o;      // (no sum that could wrap)
                if (ok) {
                    const int32_t* w = ca.schedule_words + o;
                    parts = w[3];
                    ok = w[0] == pp && w[2] == m && w[1] >= 1 && parts >= 1 && parts <= co.L && w[4] >= 1;
                    sup = sup && w[1] <= kMaxPP && parts <= kMaxPP && (int64_t)w[1] * m <= kMaxSlots;
                }
            }
        }
        ok = ok && (poff == -1 || (poff >= 0 && ca.part_pool != nullptr && poff + parts + 1 <= ca.part_pool_len));
        int v = -1;
        if (ok) {
            for (int i = co.V - 1; i >= 0; i--) if (co.variant_tp[i] == tp) v = i;
            ok = v >= 0;
        }
        if (ok && sup) {
            int k = 0;                               // class 0 = 64 lanes ... class 6 = 1 lane
            while (k < 6 && (32 >> k) >= pp) k++;
            const int mb = (m < kMBins ? m : kMBins) - 1;
            int sub = kMBins - 1 - mb;               // place in its half of the class's bins, longest first
            if (sched == 3) sub = kSubVirtual + 127 - (int)((slots3 < 2048 ? slots3 : 2047) >> 4);
            else if (sched == 4) sub = kSubExplicit + 127 - ((m < 2048 ? m : 2047) >> 4);
            else if (sched != 0) sub = m >= 1024 ? 0 : m > 512 ? (1025 - m) >> 1 : 256 + 512 - m;
            const int bin = k * kBinsPerClass + (sched != 0 ? kMBins : 0) + sub;   // ordered by sweep shape
            rank[j] = atomicAdd(&hist[bin], 1);
            key[j] = bin | (v << 24);
        } else {
            ev.num_events[c] = 0;
            ev.stage_pos[c] = -1;
        }
        ev.status[c] = ok ? (sup ? 0 : 4) : 1;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins; b += kDecodeBlock) {
        const int n = hist[b];
        if (n > 0) hist[b] = atomicAdd(&ws.bin_count[b], n);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kDecodePer; j++) {
        const int64_t c = base + (int64_t)j * kDecodeBlock;
        if (c >= C) continue;
        ws.key[c] = key[j];
        if (key[j] >= 0) ws.rank[c] = hist[key[j] & 0xffffff] + rank[j];
    }
}

// ---------------------------------------------------------------------------------------
// Ordering bins -> first position of every bin, class ranges and wave-item ranges.
constexpr int kBinsBlock = 1024;
__global__ __launch_bounds__(kBinsBlock) void k_bins(Workspace ws, int64_t stage_cap) {
    constexpr int per = kBins / kBinsBlock;
    static_assert(kBins % kBinsBlock == 0, "bins must split evenly");
    __shared__ int64_t wsum[kBinsBlock / kWave];
    __shared__ int32_t cls[kClasses + 1];
    __shared__ int32_t mid[kClasses];        // first position of each class's second half of bins (schedule != GPipe)
    const int t = threadIdx.x;
    int loc[per];
    int64_t s = 0;
    for (int i = 0; i < per; i++) { loc[i] = ws.bin_count[t * per + i]; s += loc[i]; }
    int64_t inc = wave_inclusive_sum(s);
    if (lane_id() == kWave - 1) wsum[t / kWave] = inc;
    __syncthreads();
    int64_t add = 0;
    for (int i = 0; i < t / kWave; i++) add += wsum[i];
    int64_t ex = inc - s + add;
    for (int i = 0; i < per; i++) {
        const int b = t * per + i;
        ws.bin_start[b] = (int32_t)ex;
        if (b % kBinsPerClass == 0) cls[b / kBinsPerClass] = (int32_t)ex;
        if (b % kBinsPerClass == kMBins) mid[b / kBinsPerClass] = (int32_t)ex;
        ex += loc[i];
    }
    if (t == kBinsBlock - 1) { ws.bin_start[kBins] = (int32_t)ex; cls[kClasses] = (int32_t)ex; }
    __syncthreads();
    if (t == 0) {
        int64_t items = 0;
        for (int k = 0; k < kClasses; k++) {
            const int64_t a = cls[k], b = cls[k + 1];
            ws.hdr[H_CLASS_START + k] = a;
            ws.hdr[H_ITEM_START + k] = items;
            const int64_t per_item = 1 << k;       // candidates per wave-item in class k
            // leading items of GPipe candidates only, as far as the per-stage arrays have room
            int64_t g = k < kClasses - 1 ? (mid[k] - a) >> k : 0;
            const int64_t room = stage_cap / kWave - items;
            if (g > room) g = room < 0 ? 0 : room;
            ws.hdr[H_GPIPE_ITEMS + k] = g & ~(int64_t)1;
            items += (b - a + per_item - 1) / per_item;
        }
        ws.hdr[H_CLASS_START + kClasses] = cls[kClasses];
        ws.hdr[H_ITEM_START + kClasses] = items;
        ws.hdr[H_NUM_ITEMS] = items;
    }
}

// ---------------------------------------------------------------------------------------
// Order in which the sweep kernels take the pairs of their wave-items.  Two launches share the
// items: in every class the leading items that hold only GPipe candidates (hdr[H_GPIPE_ITEMS +
// class], an even number) belong to k_simulate_gpipe, all others to k_simulate; a list of fewer
// than split_min_items wave-items is not worth two launches and goes to k_simulate whole (the host passes 0 or
// the largest integer: it decides by the number of candidates, as it does when it launches the sweeps).
// Inside a class the items are sorted by micro-batch count, longest sweep first, but the classes
// follow one another, so in visiting order the lengths form a saw-tooth: taken in that order the
// long items of the narrower classes would start late and a launch would end with a few long
// sweeps on an empty machine.  So every class is cut into kOrderGroups groups of consecutive pairs
// and a launch takes group 0 of every class, then group 1 of every class, and so on (the last
// group also holds the up to kOrderGroups - 1 pairs that the even split leaves over): pairs at the
// same relative position of their class, which have about the same micro-batch count, run at
// about the same time.  A pair never straddles two classes.
constexpr int kOrderShift = 6, kOrderGroups = 1 << kOrderShift;

// The items of class k that a launch owns: the first of them (relative to the class) and how many.
// Items past the room in the per-stage arrays (wave-item index >= item_limit) own nothing and are
// dropped from the class's end.
__device__ __forceinline__ void owned_range(const int64_t* __restrict__ hdr, int k, bool gpipe, bool split,
                                            int64_t item_limit, int32_t& first, int32_t& own) {
    const int64_t n = hdr[H_ITEM_START + k + 1] - hdr[H_ITEM_START + k], g = split ? hdr[H_GPIPE_ITEMS + k] : 0;
    const int64_t f = gpipe || !split ? 0 : g;
    int64_t o = gpipe ? g : n - g;
    const int64_t room = item_limit - hdr[H_ITEM_START + k] - f;
    if (o > room) o = room > 0 ? room : 0;
    first = (int32_t)f;
    own = (int32_t)o;
}

// Entry q of both order tables (called by thread q of k_scatter, whose grid covers order_cap).
// first_whole: the classes from this one on (the narrow ones) are taken first and whole, widest last;
// kClasses = none.  With a bucketed all-reduce the epilogue of an item walks the layers of a stage,
// so a short sweep of a stage that holds many layers is a long item all the same and must not wait
// for the end of the launch.
__device__ __forceinline__ void pair_order_entry(const Workspace& ws, int32_t q, int64_t stage_cap, int64_t split_min_items,
                                                 int first_whole) {
    const int64_t* __restrict__ hdr = ws.hdr;
    int64_t W = hdr[H_NUM_ITEMS];                       // items that have room in the per-stage arrays
    if (W * kWave > stage_cap) W = stage_cap / kWave;
    const bool split = hdr[H_NUM_ITEMS] >= split_min_items;
    for (int which = 0; which < 2; which++) {           // 0: k_simulate's pairs, 1: k_simulate_gpipe's
        const bool gpipe = which == 1;
        int32_t first[kClasses], own[kClasses], pairs[kClasses];
        int32_t group_total = 0, total = 0, whole_total = 0;
#pragma unroll
        for (int k = 0; k < kClasses; k++) {
            owned_range(hdr, k, gpipe, split, W, first[k], own[k]);       // without the split k_simulate_gpipe owns nothing
            pairs[k] = (own[k] + 1) >> 1;
            if (k >= first_whole) whole_total += pairs[k];
            else group_total += pairs[k] >> kOrderShift;
            total += pairs[k];
        }
        if (q == 0) ws.hdr[H_PAIRS + which] = total;
        if (q >= total || q >= ws.order_cap) continue;
        int32_t item = 0, has_two = 0;
        bool found = false;
        if (q < whole_total) {
            int32_t r = q;
#pragma unroll
            for (int k = kClasses - 1; k >= 0; k--) {
                if (k < first_whole) continue;
                if (!found && r < pairs[k]) {
                    found = true;
                    item = (int32_t)hdr[H_ITEM_START + k] + first[k] + 2 * r;
                    has_two = 2 * r + 1 < own[k];
                }
                if (!found) r -= pairs[k];
            }
        } else {
            const int32_t q2 = q - whole_total;
            int32_t g = kOrderGroups - 1;
            if (group_total > 0) {
                g = q2 / group_total;
                if (g > kOrderGroups - 1) g = kOrderGroups - 1;
            }
            const bool last = g == kOrderGroups - 1;
            int32_t r = q2 - g * group_total;
#pragma unroll
            for (int k = 0; k < kClasses; k++) {
                if (k >= first_whole) continue;
                const int32_t per = pairs[k] >> kOrderShift;
                const int32_t sz = last ? pairs[k] - g * per : per;
                if (!found && r < sz) {
                    found = true;
                    const int32_t j = g * per + r;
                    item = (int32_t)hdr[H_ITEM_START + k] + first[k] + 2 * j;
                    has_two = 2 * j + 1 < own[k];
                }
                if (!found) r -= sz;
            }
        }
        ws.order[which][q] = item | (has_two ? (int32_t)0x80000000 : 0);
    }
}

// Scatter candidates into visiting order and hand each its block of per-stage entries; the first
// order_cap threads also fill the order tables of the sweep kernels.
__global__ __launch_bounds__(256) void k_scatter(CandDev ca, int64_t C, Workspace ws, EventsDev ev,
                                                 int64_t split_min_items, int first_whole) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c < ws.order_cap) pair_order_entry(ws, (int32_t)c, ev.stage_cap, split_min_items, first_whole);
    if (c >= C) return;
    const int kv = ws.key[c];
    if (kv < 0) return;
    const int key = kv & 0xffffff, v = kv >> 24;
    const int k = key / kBinsPerClass;
    const int64_t pos = ws.bin_start[key] + ws.rank[c];
    const int64_t rel = pos - ws.hdr[H_CLASS_START + k];
    const int64_t item = ws.hdr[H_ITEM_START + k] + (rel >> k);
    const int64_t slot = item * kWave + ((rel & ((1 << k) - 1)) << (6 - k));
    const bool room = (item + 1) * kWave <= ev.stage_cap;
    const int pp = ca.pp[c];
    Desc d;
    d.cand = (int32_t)c;
    d.meta = (room ? pp : 0) | ((int)ca.schedule[c] << 8) | (v << 16);
    d.m = ca.m[c];
    d.dp = ca.dp[c];
    d.poff = ca.part_off[c];
    d.spare = (int64_t)ca.tp[c] | ((int64_t)(ca.chunks ? ca.chunks[c] : 1) << 32);   // tp | chunks << 32
    ws.desc[pos] = d;
    ev.stage_pos[c] = room ? slot : -1;
    if (!room) { ev.status[c] = 3; ev.num_events[c] = 0; }
}

// ---------------------------------------------------------------------------------------
// Per-stage composed events.  Lane (g, s) of a wave-item handles stage s of the g-th candidate
// of the item: the stage's layer events are reduced with prefix differences over the layer
// axis (segmented sums), the p2p events of its two boundaries and its gradient all-reduce are
// evaluated, and the row is written to the stage table (64 consecutive entries per wave and
// column).  The partition check and the 2^53 guard are group reductions over the stages.
// Per-stage composed events of one lane = (candidate, stage s).
struct StageRow {
    int64_t FC, FA, BC, BA;     // forward / backward computation and in-stage communication
    int64_t PF, PB;             // p2p events towards stage s+1 / s-1
    int64_t G;                  // gradient bytes
};

// Reduces the layer events of the lane's stage with prefix differences over the layer axis
// (segmented sums), looks up the p2p events of its two boundaries, checks the partition and
// applies the 2^53 guard (both are reductions over the candidate's lanes).  Every lane of the
// wavefront must call it.  Returns 0, or the status of a candidate that must be dropped
// (1 = not a partition, 2 = range); rows of dropped candidates and of idle lanes are zero.
// Partition check and link classes of one stage: returns nonzero when the candidate's layer
// bounds are not a partition of [0, L) (a reduction over the candidate's lanes); inter_next /
// inter_prev say whether the p2p to the next / previous stage crosses nodes, read off the row's
// mask of inter-node boundaries (k_layer_tables; row0 = first entry of the candidate's (variant, pp)
// row of Workspace::comb, looked at by the lanes that hold a stage only).
__device__ __forceinline__ int stage_check(const int64_t* row0, int L, int width, int s, int pp,
                                           int lo, int hi, int& inter_next, int& inter_prev) {
    int bad = 0;
    inter_next = 0; inter_prev = 0;
    if (s < pp) {
        bad = (hi <= lo) || (hi > L) || (s == 0 && lo != 0) || (s == pp - 1 && hi != L);
        const uint64_t mask = (uint64_t)row0[4];
        inter_next = (int)((mask >> s) & 1);
        inter_prev = (int)(((mask << 1) >> s) & 1);
    }
    return group_any(bad != 0, width) ? 1 : 0;
}

// The 2^53 guard: every timestamp of the pipeline phase is bounded by m * (all task and p2p
// durations of the candidate); per_stage is this lane's share of that sum.
__device__ __forceinline__ bool stage_out_of_range(int64_t per_stage, int m, int width) {
    // a cheap sufficient test first: if width * m * (a lane's share) stays below 2^53 in every
    // lane, so does m * (sum of the shares); only otherwise the sum itself is formed
    const uint64_t v = (uint64_t)per_stage;
    const bool small = (v >> 32) == 0 && (uint64_t)(uint32_t)v * (uint32_t)(m * width) < (1ull << 53);
    if (__builtin_amdgcn_ballot_w64(!small) == 0) return false;     // the usual case, decided for the whole wavefront
    const uint64_t t1 = (uint64_t)group_sum(per_stage, width);
    return __umul64hi(t1, (uint64_t)m) != 0 || t1 * (uint64_t)m >= (1ull << 53);
}

__device__ __forceinline__ int stage_row(const ClusterDev& cl, const Workspace& ws, int L, int width, int s,
                                         int pp, int v, int m, int dp, int tp, int lo, int hi, StageRow& r) {
    r = StageRow{0, 0, 0, 0, 0, 0, 0};
    int inter_next, inter_prev;
    const int bad = stage_check(ws.comb + (size_t)((v * kMaxPP + pp - 1) * (L + 1)) * kCombWords, L, width, s, pp, lo, hi,
                                inter_next, inter_prev);
    if (s < pp && !bad) {
        const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
        r.FC = ws.pfc[vr + hi] - ws.pfc[vr + lo];
        r.BC = ws.pbc[vr + hi] - ws.pbc[vr + lo];
        r.FA = ws.pfa[rr + hi] - ws.pfa[rr + lo];
        r.BA = ws.pba[rr + hi] - ws.pba[rr + lo];
        r.G = ws.pg[vr + hi] - ws.pg[vr + lo];
        if (s + 1 < pp) r.PF = ws.p2p[((size_t)v * L + hi - 1) * 2 + inter_next];
        if (s > 0) r.PB = ws.p2p[((size_t)v * L + lo - 1) * 2 + inter_prev];
    }
    const bool range = stage_out_of_range(r.FC + r.FA + r.BC + r.BA + r.PF + r.PB, m, width);
    const int drop = bad ? 1 : (range ? 2 : 0);
    if (drop) r = StageRow{0, 0, 0, 0, 0, 0, 0};
    return drop;
}

// What simulate needs of a stage's composed events: duration of the forward and of the backward
// stage-task without p2p (computation + in-stage communication), the computation of both, the
// gradient bytes and the two outgoing p2p events.  Same contract as stage_row, fed from
// Workspace::comb.
struct StageSums {
    int64_t FT, BT, CP, G, PF, PB;
    double inv_ar;              // 1 / (dp * beta) of the gradient all-reduce over the row's dp group
};

__device__ __forceinline__ int stage_sums(const ClusterDev& cl, const Workspace& ws, int L, int width, int s,
                                          int pp, int v, int m, int dp, int tp, int lo, int hi, StageSums& r) {
    r = StageSums{0, 0, 0, 0, 0, 0, 0.0};
    int inter_next, inter_prev;
    const int64_t* row = ws.comb + (size_t)((v * kMaxPP + pp - 1) * (L + 1)) * kCombWords;
    const int bad = stage_check(row, L, width, s, pp, lo, hi, inter_next, inter_prev);
    if (s < pp && !bad) {
        r.inv_ar = __longlong_as_double(row[5]);
        const longlong2* e_hi = (const longlong2*)(row + hi * kCombWords);
        const longlong2* e_lo = (const longlong2*)(row + lo * kCombWords);
        const longlong2 h0 = e_hi[0], h1 = e_hi[1], l0 = e_lo[0], l1 = e_lo[1];
        r.FT = h0.x - l0.x;
        r.BT = h0.y - l0.y;
        r.CP = h1.x - l1.x;
        r.G = h1.y - l1.y;
        if (s + 1 < pp) r.PF = row[hi * kCombWords + 4 + inter_next];
        if (s > 0) r.PB = row[lo * kCombWords + 4 + inter_prev];
    }
    const bool range = stage_out_of_range(r.FT + r.BT + r.PF + r.PB, m, width);
    const int drop = bad ? 1 : (range ? 2 : 0);
    // rare: the branch is taken by the whole wavefront or not at all
    if (__builtin_amdgcn_ballot_w64(drop != 0) != 0) {
        if (drop) r = StageSums{0, 0, 0, 0, 0, 0, 0.0};
    }
    return drop;
}

// Number of gradient all-reduce events on the stage's device (data-parallel modelling).
__device__ __forceinline__ int64_t count_allreduce_events(const ClusterDev& cl, const Workspace& ws, int L, int v,
                                                          int dp, int lo, int hi, int64_t G) {
    if (dp <= 1 || G <= 0) return 0;
    if (cl.bucket <= 0) return 1;
    const size_t vr = (size_t)v * (L + 1);
    int64_t acc = 0, n = 0;
    for (int l = hi - 1; l >= lo; l--) {
        acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
        const int64_t k = (int64_t)udiv64((uint64_t)acc, (uint64_t)cl.bucket);
        n += k;
        acc -= k * cl.bucket;
    }
    return n + (acc > 0 ? 1 : 0);
}

// The descriptor of the wave's next item and that item's partition bytes are requested one
// iteration ahead, so that an item's own chain of dependent loads is only tables -> stores.
struct StageWork {
    int sh, s;
    int64_t pos;
    Desc d;
    int lo, hi;
};

__device__ __forceinline__ void stage_fetch_desc(const Workspace& ws, const int64_t* hdr, int64_t w, int lane,
                                                 StageWork& x) {
    const Item it = decode_item(hdr, w);
    x.sh = it.sh;
    x.s = lane & ((1 << it.sh) - 1);
    x.pos = it.pos0 + (lane >> it.sh);
    x.d = Desc{};
    if (x.pos < it.class_end) x.d = ws.desc[x.pos];
    if (has_own_kernel(x.d)) x.d = Desc{};
}

__device__ __forceinline__ void stage_fetch_bounds(const CandDev& ca, int L, StageWork& x) {
    const int pp = x.d.meta & 0xff;
    x.lo = 0; x.hi = 0;
    if (x.s < pp) {
        if (x.d.poff >= 0) { x.lo = ca.part_pool[x.d.poff + x.s]; x.hi = ca.part_pool[x.d.poff + x.s + 1]; }
        else { x.lo = uniform_bound(x.s, L, pp); x.hi = uniform_bound((x.s + 1), L, pp); }
    }
}

// Writes the per-stage composed events of every candidate to the stage table (64 consecutive
// entries per wavefront and column).  Optional: distsim_simulate regenerates the rows itself.
__global__ __launch_bounds__(256) void k_stage_events(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                      EventsDev ev) {
    const int lane = lane_id();
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    __shared__ int64_t hdr[H_WORDS];
    if (threadIdx.x < H_WORDS) hdr[threadIdx.x] = ws.hdr[threadIdx.x];
    __syncthreads();
    int64_t W = hdr[H_NUM_ITEMS];
    if (W * kWave > ev.stage_cap) W = ev.stage_cap / kWave;       // items beyond the capacity own nothing
    const int L = co.L;
    const int64_t cap = ev.stage_cap;
    StageWork nx{};
    if (wave0 < W) { stage_fetch_desc(ws, hdr, wave0, lane, nx); stage_fetch_bounds(ca, L, nx); }
    for (int64_t w = wave0; w < W; w += nwaves) {
        const StageWork cur = nx;
        const bool more = w + nwaves < W;
        if (more) stage_fetch_desc(ws, hdr, w + nwaves, lane, nx);
        const int width = 1 << cur.sh;
        const int s = cur.s;
        const Desc d = cur.d;
        const int pp = d.meta & 0xff, v = d.meta >> 16, m = d.m, dp = d.meta ? d.dp : 1;
        const bool act = s < pp;
        StageRow r;
        const int drop = stage_row(cl, ws, L, width, s, pp, v, m, dp, (int)d.spare, cur.lo, cur.hi, r);
        const bool sync = ((d.meta >> 8) & 0xff) != 2;      // the asynchronous schedule has no gradient all-reduce
        const int64_t AR = sync ? allreduce_ns(cl, dp, r.G) : 0;
        int64_t nar = (act && !drop && sync) ? count_allreduce_events(cl, ws, L, v, dp, cur.lo, cur.hi, r.G) : 0;
        if (more) stage_fetch_bounds(ca, L, nx);
        nar = group_sum(nar, width);
        const int lo_w = drop ? 0 : cur.lo, hi_w = drop ? 0 : cur.hi;
        const int64_t i = w * kWave + lane;
        // written once and not read again by the library: streaming stores
        __builtin_nontemporal_store(r.FC, &ev.stage_tab[0 * cap + i]);
        __builtin_nontemporal_store(r.FA, &ev.stage_tab[1 * cap + i]);
        __builtin_nontemporal_store(r.BC, &ev.stage_tab[2 * cap + i]);
        __builtin_nontemporal_store(r.BA, &ev.stage_tab[3 * cap + i]);
        __builtin_nontemporal_store(r.PF, &ev.stage_tab[4 * cap + i]);
        __builtin_nontemporal_store(r.PB, &ev.stage_tab[5 * cap + i]);
        __builtin_nontemporal_store(r.G, &ev.stage_tab[6 * cap + i]);
        __builtin_nontemporal_store(AR, &ev.stage_tab[7 * cap + i]);
        __builtin_nontemporal_store((int32_t)(lo_w | (hi_w << 8)), &ev.stage_layers[i]);
        if (act && s == 0) {
            const int64_t c = d.cand;
            if (drop) {
                ev.status[c] = drop;
                ev.num_events[c] = 0;
            } else {
                ev.num_events[c] = 2ll * m * pp + 2ll * m * (pp - 1) + nar;
            }
        }
    }
}

}  // namespace distsim
