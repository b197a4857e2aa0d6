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
};

// One wave-item = 64 lanes = (64 >> sh) consecutive candidates of one class, 1 << sh lanes each.
struct Item {
    int sh;
    int64_t pos0, class_end;
};

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
// same event (Sec. 3.2).
__global__ __launch_bounds__(64) void k_layer_tables(CostsDev co, ClusterDev cl, Workspace ws) {
    const int row = blockIdx.x;
    const int v = row / kMaxPP, pp = row % kMaxPP + 1;
    const int lane = threadIdx.x;
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
    int64_t c_fa = 0, c_ba = 0, c_fc = 0, c_bc = 0, c_g = 0;
    if (lane == 0) {
        pfa[0] = 0; pba[0] = 0;
        if (base) { pfc[0] = 0; pbc[0] = 0; pg[0] = 0; }
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
        if (in) { pfa[l + 1] = f; pba[l + 1] = b; }
        c_fa = __shfl(f, kWave - 1, kWave);
        c_ba = __shfl(b, kWave - 1, kWave);
        if (base) {
            int64_t a = wave_inclusive_sum(in ? co.fc[i] : 0) + c_fc;
            int64_t bb = wave_inclusive_sum(in ? co.bc[i] : 0) + c_bc;
            int64_t g = wave_inclusive_sum(in ? co.grad[i] : 0) + c_g;
            if (in) { pfc[l + 1] = a; pbc[l + 1] = bb; pg[l + 1] = g; }
            c_fc = __shfl(a, kWave - 1, kWave);
            c_bc = __shfl(bb, kWave - 1, kWave);
            c_g = __shfl(g, kWave - 1, kWave);
        }
    }
}

__global__ void k_clear_bins(Workspace ws) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < kBins) { ws.bin_count[i] = 0; ws.bin_fill[i] = 0; }
}

__device__ __forceinline__ int boundary_class(const ClusterDev& cl, int64_t tpdp, int s) {
    const int64_t g = cl.gpus_per_node;
    return ((int64_t)s * tpdp) / g == ((int64_t)(s + 1) * tpdp) / g ? 0 : 1;
}

// ---------------------------------------------------------------------------------------
// Candidate decoding: one thread per candidate.  Validates the strategy, applies the 2^53
// range guard, and files the candidate into its ordering bin.
__global__ __launch_bounds__(256) void k_decode(CostsDev co, ClusterDev cl, CandDev ca, int64_t C,
                                                Workspace ws, int32_t* __restrict__ status,
                                                int64_t* __restrict__ num_events) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const int L = co.L;
    const int32_t dp = ca.dp[c], tp = ca.tp[c], pp = ca.pp[c], m = ca.m[c];
    const int sched = ca.schedule[c];
    const int64_t poff = ca.part_off[c];
    bool ok = dp >= 1 && tp >= 1 && pp >= 1 && m >= 1 && m <= kMaxM && sched <= 1 && pp <= L && pp <= kMaxPP;
    ok = ok && (int64_t)dp * tp * pp == (int64_t)cl.num_devices;
    int v = -1;
    if (ok) {
        for (int i = co.V - 1; i >= 0; i--) if (co.variant_tp[i] == tp) v = i;
        ok = v >= 0;
    }
    const uint8_t* bnd = nullptr;
    if (ok && poff != -1) {
        ok = poff >= 0 && ca.part_pool != nullptr && poff + pp + 1 <= ca.part_pool_len;
        if (ok) {
            bnd = ca.part_pool + poff;
            ok = bnd[0] == 0 && bnd[pp] == L;
            for (int s = 0; s < pp && ok; s++) ok = bnd[s + 1] > bnd[s];
        }
    }
    int st = ok ? 0 : 1;
    if (ok) {
        // every timestamp of the pipeline phase is bounded by m * (all task + p2p durations)
        const int row = v * kMaxPP + (pp - 1);
        uint64_t t1 = (uint64_t)ws.pfc[(size_t)v * (L + 1) + L] + (uint64_t)ws.pbc[(size_t)v * (L + 1) + L] +
                      (uint64_t)ws.pfa[(size_t)row * (L + 1) + L] + (uint64_t)ws.pba[(size_t)row * (L + 1) + L];
        const int64_t tpdp = (int64_t)tp * dp;
        for (int s = 0; s + 1 < pp; s++) {
            const int last = bnd ? bnd[s + 1] - 1 : (int)(((int64_t)(s + 1) * L) / pp) - 1;
            t1 += 2ull * (uint64_t)p2p_ns(cl, co.act[(size_t)v * L + last], boundary_class(cl, tpdp, s));
        }
        if (t1 > ((1ull << 53) - 1) / (uint64_t)m) st = 2;
    }
    status[c] = st;
    int key = -1;
    if (st == 0) {
        int k = 0;                                   // class 0 = 64 lanes ... class 6 = 1 lane
        while (k < 6 && (32 >> k) >= pp) k++;
        const int mb = (m < kMBins ? m : kMBins) - 1;
        key = k * kBinsPerClass + sched * kMBins + (kMBins - 1 - mb);
        atomicAdd(&ws.bin_count[key], 1);
    } else {
        num_events[c] = 0;
    }
    ws.npp[c] = st == 0 ? pp : 0;
    ws.key[c] = st == 0 ? (key | (v << 24)) : -1;
}

// ---------------------------------------------------------------------------------------
// Exclusive prefix sum of npp -> stage_off (three small kernels).
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t v, int64_t* total) {
    __shared__ int64_t wsum[kScanBlock / kWave];
    const int lane = lane_id(), wv = threadIdx.x / kWave;
    int64_t inc = wave_inclusive_sum(v);
    if (lane == kWave - 1) wsum[wv] = inc;
    __syncthreads();
    int64_t add = 0, tot = 0;
    for (int i = 0; i < kScanBlock / kWave; i++) {
        if (i < wv) add += wsum[i];
        tot += wsum[i];
    }
    __syncthreads();
    *total = tot;
    return inc - v + add;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_reduce(const int32_t* __restrict__ npp, int64_t C,
                                                             int64_t* __restrict__ block_sums) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int64_t s = 0;
    for (int i = 0; i < kScanItems; i++) if (base + i < C) s += npp[base + i];
    int64_t tot;
    block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_top(int64_t* __restrict__ block_sums, int64_t nblocks) {
    int64_t carry = 0;
    for (int64_t b0 = 0; b0 < nblocks; b0 += kScanBlock) {
        const int64_t i = b0 + threadIdx.x;
        const int64_t v = i < nblocks ? block_sums[i] : 0;
        int64_t tot;
        const int64_t ex = block_exclusive_scan(v, &tot);
        if (i < nblocks) block_sums[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) block_sums[nblocks] = carry;
}

__global__ __launch_bounds__(kScanBlock) void k_scan_apply(const int32_t* __restrict__ npp, int64_t C,
                                                            const int64_t* __restrict__ block_sums,
                                                            int64_t nblocks, int64_t* __restrict__ stage_off) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int64_t v[kScanItems], s = 0;
    for (int i = 0; i < kScanItems; i++) { v[i] = base + i < C ? npp[base + i] : 0; s += v[i]; }
    int64_t tot;
    int64_t ex = block_exclusive_scan(s, &tot) + block_sums[blockIdx.x];
    for (int i = 0; i < kScanItems; i++) {
        if (base + i < C) stage_off[base + i] = ex;
        ex += v[i];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) stage_off[C] = block_sums[nblocks];
}

// ---------------------------------------------------------------------------------------
// Ordering bins -> first position of every bin, class ranges and wave-item ranges.
constexpr int kBinsBlock = 1024;
__global__ __launch_bounds__(kBinsBlock) void k_bins(Workspace ws) {
    constexpr int per = kBins / kBinsBlock;
    static_assert(kBins % kBinsBlock == 0, "bins must split evenly");
    __shared__ int64_t wsum[kBinsBlock / kWave];
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
    for (int i = 0; i < per; i++) { ws.bin_start[t * per + i] = (int32_t)ex; ex += loc[i]; }
    if (t == kBinsBlock - 1) ws.bin_start[kBins] = (int32_t)ex;
    __syncthreads();
    __threadfence_block();
    if (t == 0) {
        int64_t items = 0;
        for (int k = 0; k < kClasses; k++) {
            // bin_start entries at class boundaries were written by other threads of this block
            const int64_t a = ((volatile int32_t*)ws.bin_start)[k * kBinsPerClass];
            const int64_t b = ((volatile int32_t*)ws.bin_start)[(k + 1) * kBinsPerClass];
            ws.hdr[H_CLASS_START + k] = a;
            ws.hdr[H_ITEM_START + k] = items;
            const int64_t per_item = 1 << k;       // candidates per wave-item in class k
            items += (b - a + per_item - 1) / per_item;
            if (k == kClasses - 1) ws.hdr[H_CLASS_START + kClasses] = b;
        }
        ws.hdr[H_ITEM_START + kClasses] = items;
        ws.hdr[H_NUM_ITEMS] = items;
    }
}

// Scatter candidates into visiting order.
__global__ __launch_bounds__(256) void k_scatter(CandDev ca, int64_t C, Workspace ws, int64_t stage_cap,
                                                 const int64_t* __restrict__ stage_off,
                                                 int32_t* __restrict__ status, int64_t* __restrict__ num_events) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const int kv = ws.key[c];
    if (kv < 0) return;
    const int key = kv & 0xffffff, v = kv >> 24;
    const int pos = ws.bin_start[key] + atomicAdd(&ws.bin_fill[key], 1);
    const int pp = ca.pp[c];
    const int64_t off = stage_off[c];
    const bool room = off + pp <= stage_cap;
    if (!room) { status[c] = 3; num_events[c] = 0; }
    ws.s_cand[pos] = (int32_t)c;
    ws.s_meta[pos] = (room ? pp : 0) | ((int)ca.schedule[c] << 8) | (v << 16);
    ws.s_m[pos] = ca.m[c];
    ws.s_dp[pos] = ca.dp[c];
    ws.s_off[pos] = off;
}

// ---------------------------------------------------------------------------------------
// Per-stage composed events.  Lane (g, s) of a wave-item handles stage s of the g-th candidate
// of the item: the stage's layer events are reduced with prefix differences over the layer
// axis (segmented sums), the p2p events of its two boundaries and its gradient all-reduce are
// evaluated, and the row is written to the stage table.
struct EventsDev {
    int64_t stage_cap;
    int64_t* stage_tab;
    int32_t* stage_layers;
    int64_t* num_events;
};

__global__ __launch_bounds__(256) void k_stage_events(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                      EventsDev ev) {
    const int lane = lane_id();
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    const int64_t W = ws.hdr[H_NUM_ITEMS];
    const int L = co.L;
    for (int64_t w = wave0; w < W; w += nwaves) {
        const Item it = decode_item(ws.hdr, w);
        const int width = 1 << it.sh;
        const int s = lane & (width - 1);
        const int64_t pos = it.pos0 + (lane >> it.sh);
        int pp = 0, v = 0, m = 0, dp = 1;
        int64_t off = 0, c = 0;
        if (pos < it.class_end) {
            const int meta = ws.s_meta[pos];
            pp = meta & 0xff; v = meta >> 16;
            m = ws.s_m[pos]; dp = ws.s_dp[pos];
            off = ws.s_off[pos]; c = ws.s_cand[pos];
        }
        const bool act = s < pp;
        int64_t nar = 0;
        if (act) {
            const int64_t poff = ca.part_off[c];
            int lo, hi;
            if (poff >= 0) { lo = ca.part_pool[poff + s]; hi = ca.part_pool[poff + s + 1]; }
            else { lo = (int)(((int64_t)s * L) / pp); hi = (int)(((int64_t)(s + 1) * L) / pp); }
            const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
            const int tp = co.variant_tp[v];
            const int64_t tpdp = (int64_t)tp * dp;
            const int64_t FC = ws.pfc[vr + hi] - ws.pfc[vr + lo];
            const int64_t BC = ws.pbc[vr + hi] - ws.pbc[vr + lo];
            const int64_t FA = ws.pfa[rr + hi] - ws.pfa[rr + lo];
            const int64_t BA = ws.pba[rr + hi] - ws.pba[rr + lo];
            const int64_t G = ws.pg[vr + hi] - ws.pg[vr + lo];
            int64_t PF = 0, PB = 0;
            if (s + 1 < pp) PF = p2p_ns(cl, co.act[(size_t)v * L + hi - 1], boundary_class(cl, tpdp, s));
            if (s > 0) PB = p2p_ns(cl, co.act[(size_t)v * L + lo - 1], boundary_class(cl, tpdp, s - 1));
            const int64_t AR = allreduce_ns(cl, dp, G);
            const int64_t i = off + s;
            const int64_t cap = ev.stage_cap;
            ev.stage_tab[0 * cap + i] = FC;
            ev.stage_tab[1 * cap + i] = FA;
            ev.stage_tab[2 * cap + i] = BC;
            ev.stage_tab[3 * cap + i] = BA;
            ev.stage_tab[4 * cap + i] = PF;
            ev.stage_tab[5 * cap + i] = PB;
            ev.stage_tab[6 * cap + i] = G;
            ev.stage_tab[7 * cap + i] = AR;
            ev.stage_layers[i] = lo | (hi << 8);
            // gradient all-reduce events on this stage's device
            if (dp > 1 && G > 0) {
                if (cl.bucket <= 0) {
                    nar = 1;
                } else {
                    int64_t acc = 0;
                    for (int l = hi - 1; l >= lo; l--) {
                        acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
                        const int64_t k = acc / cl.bucket;
                        nar += k;
                        acc -= k * cl.bucket;
                    }
                    if (acc > 0) nar += 1;
                }
            }
        }
        nar = group_sum(nar, width);
        if (act && s == 0)
            ev.num_events[c] = 2ll * m * pp + 2ll * m * (pp - 1) + nar;
    }
}

}  // namespace distsim
