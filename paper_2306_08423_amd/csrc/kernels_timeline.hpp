// Timeline dump: start and end of every stage-task of selected candidates, i.e. the per-device
// event lists of Algorithm 1 reduced to their stage-tasks, plus the window of the gradient
// all-reduce events of every stage (Sec. 3.2: the timeline says at what time which device computes
// or communicates).
#pragma once
#include "kernels_simulate.hpp"

namespace distsim {

struct TimelineOut {
    const int64_t* sel;         // [n] candidate indices
    const int64_t* task_off;    // [n] first entry of the candidate's block in start / end
    int64_t* start;             // block layout [2][pp][m]: kind (0 forward, 1 backward), stage, micro-batch
    int64_t* end;
    int64_t* ar_start;          // [n][kMaxPP] start of the stage's first all-reduce event, -1 = none
    int64_t* ar_end;            // [n][kMaxPP] end of its last one
};

// A row of the staging ring takes the entries of kTlFlush levels plus what the last flush left
// behind because it did not fill an aligned group of kTlFlush entries (32 bytes).
constexpr int kTlFlush = 4;              // levels between two flushes = entries per aligned write
constexpr int kTlRing = 2 * kTlFlush;    // ring capacity per row
constexpr int kTlRow = kTlRing + 1;      // padded: consecutive stages start in different LDS banks
constexpr int kTlChunk = 16;             // selected candidates per workgroup (at most 64)
constexpr int kTlWaves = 4;
static_assert(kTlChunk <= kWave && kTlWaves >= 1, "one wavefront sorts a chunk; blocks are kTlWaves whole wavefronts");

// Per-wavefront staging area.
struct TlRowMeta { int64_t base, dur; };     // index of the row's entry 0 in start / end; task duration
struct TlStage {
    double ring[2][kWave][kTlRow];           // start times of the newest tasks, [kind][lane][micro-batch mod kTlRing]
    TlRowMeta meta[2][kWave];
    int2 span[2][kWave];                     // entries [x, y) of the row that the running flush writes
};

// A workgroup takes kTlChunk consecutive entries of the selection, sorts them by the number of
// lanes they need (64, 32, ... 1) and packs them into wave-items like simulate does, so that
// candidates with few stages share a wavefront; its four wavefronts take the items in turn.
// The sweep is the level sweep of kernels_simulate.hpp (same level functions, bit patterns and
// task step) with one addition: after each step the lanes that ran a task put its start time
// into an LDS ring, one row per (kind, lane).  A stage's tasks of one kind come in micro-batch
// order, so what a row gains between two flushes is one run of consecutive micro-batches; every
// kTlFlush levels the wavefront writes out, per row, the entries up to the last 32-byte boundary
// of the output arrays (the rest waits for the next flush; the last flush writes everything),
// kTlFlush lanes per row and 64 / kTlFlush rows per store: whole aligned sectors instead of one
// partial cache line per lane.  The end time is the start plus the row's task duration.  The staging area belongs to one
// wavefront, whose LDS instructions execute in order: between its writes and the reads by other
// lanes only the compiler has to be kept from reordering (wavefront-scope fences).
__global__ __launch_bounds__(kTlWaves * kWave) void k_timeline(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                               const int32_t* __restrict__ status, int64_t C,
                                                               int64_t n, TimelineOut out) {
    __shared__ TlStage stage_mem[kTlWaves];
    __shared__ int32_t order[kTlChunk];
    __shared__ int32_t cls_start[kClasses + 1], cls_count[kClasses], item_start[kClasses + 1];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t q0 = (int64_t)blockIdx.x * kTlChunk;
    const int L = co.L;

    // all-reduce windows default to "none"
    for (int i = threadIdx.x; i < kTlChunk * kMaxPP; i += blockDim.x) {
        const int64_t q = q0 + i / kMaxPP;
        if (q < n) { out.ar_start[q * kMaxPP + i % kMaxPP] = -1; out.ar_end[q * kMaxPP + i % kMaxPP] = -1; }
    }
    // counting sort of the chunk by width class (first wavefront)
    if (wave == 0) {
        const int64_t q = q0 + lane;
        int k = -1;
        if (lane < kTlChunk && q < n) {
            const int64_t c = out.sel[q];
            if (c >= 0 && c < C && status[c] == 0 && ca.schedule[c] < 3) {       // the interleaved schedule has a dump of its own, explicit ones none
                const int pp = ca.pp[c];
                int sh = 0;
                while ((1 << sh) < pp) sh++;
                k = 6 - sh;
            }
        }
        int at = 0, items = 0;
        for (int kk = 0; kk < kClasses; kk++) {
            const uint64_t b = __builtin_amdgcn_ballot_w64(k == kk);
            const int cnt = __popcll(b);
            if (k == kk) order[at + __popcll(b & ((1ull << lane) - 1))] = lane;
            if (lane == 0) { cls_start[kk] = at; cls_count[kk] = cnt; item_start[kk] = items; }
            at += cnt;
            items += (cnt + (1 << kk) - 1) >> kk;
        }
        if (lane == 0) { cls_start[kClasses] = at; item_start[kClasses] = items; }
    }
    __syncthreads();

    TlStage& sm = stage_mem[wave];
    const double ninf = -__builtin_huge_val();
    const int total_items = item_start[kClasses];
    for (int w = wave; w < total_items; w += kTlWaves) {
        int k = 0;
        while (w >= item_start[k + 1]) k++;
        const int sh = 6 - k, width = 1 << sh;
        const int g = lane >> sh, s = lane & (width - 1);
        const int slot = ((w - item_start[k]) << k) + g;          // position inside the class
        const bool have = slot < cls_count[k];
        const int64_t q = q0 + (have ? order[cls_start[k] + slot] : 0);
        const int64_t c = have ? out.sel[q] : 0;
        int pp = 0, m = 0, dp = 1, tp = 1, sched = 0;
        int64_t poff = -1;
        if (have) { pp = ca.pp[c]; m = ca.m[c]; dp = ca.dp[c]; tp = ca.tp[c]; sched = ca.schedule[c]; poff = ca.part_off[c]; }
        int v = 0;
        for (int i = co.V - 1; i >= 0; i--) if (co.variant_tp[i] == tp) v = i;
        bool act = s < pp;
        int lo = 0, hi = 0;
        if (act) {
            if (poff >= 0) { lo = ca.part_pool[poff + s]; hi = ca.part_pool[poff + s + 1]; }
            else { lo = uniform_bound(s, L, pp); hi = uniform_bound((s + 1), L, pp); }
        }
        StageRow r;
        // a candidate whose partition or range check fails gets no entries
        if (stage_row(cl, ws, L, width, s, pp, v, m, dp, tp, lo, hi, r) != 0) act = false;
        if (!act) { pp = 0; m = 0; }
        const int64_t pf_task = cl.blocking == 1 ? r.PF : 0, pb_task = cl.blocking == 1 ? r.PB : 0;
        const int64_t Fd_i = r.FC + r.FA + pf_task, Bd_i = r.BC + r.BA + pb_task;
        const double Fd = (double)Fd_i, Bd = (double)Bd_i;
        double pfL = from_prev_lane((double)(r.PF - pf_task)), pbR = from_next_lane((double)(r.PB - pb_task));
        if (!(act && s > 0)) pfL = ninf;
        if (!(act && s + 1 < pp)) pbR = ninf;
        const int64_t off = act ? out.task_off[q] : 0;
        const int64_t baseF = off + (int64_t)s * m, baseB = off + ((int64_t)pp + s) * m;   // rows [kind][stage][0]
        sm.meta[0][lane] = TlRowMeta{baseF, Fd_i};
        sm.meta[1][lane] = TlRowMeta{baseB, Bd_i};

        // level windows of this lane on x = level - s (see kernels_simulate.hpp)
        int f1hi, f2lo = 1, f2hi = 0, blo, bhi;
        if (sched == 0) {
            f1hi = m - 1;
            blo = m + 2 * pp - 2 - 2 * s; bhi = blo + m - 1;
        } else {
            int wq = pp - 1 - s; if (wq > m) wq = m;
            f1hi = wq < m - 1 ? wq : m - 1;
            f2lo = 2 * wq + 2; f2hi = 2 * m - 2;
            blo = 2 * pp - 1 - 2 * s; bhi = blo + 2 * m - 2;
        }
        const int nlev = wave_max_i32(act ? 2 * (m + pp - 1) : 0);
        double own = 0.0;
        double linkF = 0.0, linkB = 0.0;                      // p2p_blocking = 2: arrival of the lane's latest sends
        const double sendF = (double)r.PF, sendB = (double)r.PB;
        const bool hasL = act && s > 0, hasR = act && s + 1 < pp;
        int nF = 0, nB = 0, fF = 0, fB = 0;                   // tasks run / written out, per kind
        uint64_t kmask = 0, kmask2 = 0;
        for (int l0 = 0; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;
            uint32_t PFb = level_bits(-x0, f1hi - x0) | (level_bits(f2lo - x0, f2hi - x0) & even_x);
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            if (sched != 0) PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;
            if (!act) { PFb = 0; PBb = 0; }
            const bool anyF = wave_or_u32(PFb) != 0, anyB = wave_or_u32(PBb) != 0;
            const int kend = nlev - l0 < 32 ? nlev - l0 : 32;
            for (int kk = 0; kk < kend; kk++) {
                bool ranF = false, ranB = false;                 // this lane ran a forward / backward task
                double tF = 0.0, tB = 0.0;                       // and it started at
                if (cl.blocking == 2) {
                    // sends queue on their link: the neighbour reads the arrival time of the send
                    const double arrL = from_prev_lane(linkF), arrR = from_next_lane(linkB);
                    if (PFb >> 31) {
                        tF = hasL && arrL > own ? arrL : own;
                        own = tF + Fd;
                        if (hasR) linkF = (own > linkF ? own : linkF) + sendF;
                        ranF = true;
                    } else if (PBb >> 31) {
                        tB = hasR && arrR > own ? arrR : own;
                        own = tB + Bd;
                        if (hasL) linkB = (own > linkB ? own : linkB) + sendB;
                        ranB = true;
                    }
                    PFb <<= 1; PBb <<= 1;
                } else if (anyF && anyB) {
                    double tl = from_prev_lane(own), tr = from_next_lane(own);
                    DISTSIM_STEPFB1(PFb, PBb, own, tl, tr, pfL, pbR, Fd, Bd);
                    ranF = (kmask >> lane) & 1; tF = tl;
                    ranB = (kmask2 >> lane) & 1; tB = tr;
                } else if (anyF) {
                    double tl = from_prev_lane(own);
                    DISTSIM_STEP1(PFb, own, tl, pfL, Fd);
                    ranF = (kmask >> lane) & 1; tF = tl;
                } else if (anyB) {
                    double tr = from_next_lane(own);
                    DISTSIM_STEP1(PBb, own, tr, pbR, Bd);
                    ranB = (kmask >> lane) & 1; tB = tr;
                }
                if (ranF) { sm.ring[0][lane][nF & (kTlRing - 1)] = tF; nF++; }
                if (ranB) { sm.ring[1][lane][nB & (kTlRing - 1)] = tB; nB++; }
                const bool last = l0 + kk == nlev - 1;
                if ((kk & (kTlFlush - 1)) != kTlFlush - 1 && !last) continue;
                // flush: per row the entries [flushed, upto), upto = done rounded down to a sector
                // boundary of the output (done itself in the last flush, which may take two rounds)
                constexpr int kGroups = kTlFlush, kRowsPer = kWave / kTlFlush;   // stores per kind, rows per store
                for (int round = 0; round < (last ? 2 : 1); round++) {
                    int upF = last ? nF : nF - (int)((baseF + nF) & (kTlFlush - 1));
                    int upB = last ? nB : nB - (int)((baseB + nB) & (kTlFlush - 1));
                    if (upF > fF + kTlFlush) upF = fF + kTlFlush;
                    if (upB > fB + kTlFlush) upB = fB + kTlFlush;
                    sm.span[0][lane] = make_int2(fF, upF);
                    sm.span[1][lane] = make_int2(fB, upB);
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    const int rsub = lane / kTlFlush, e = lane & (kTlFlush - 1);
                    for (int kind = 0; kind < 2; kind++) {
                        if (__builtin_amdgcn_ballot_w64(kind ? upB > fB : upF > fF) == 0) continue;
                        // all LDS reads of the kGroups stores first, then the stores
                        int2 sp[kGroups];
                        TlRowMeta mt[kGroups];
                        double val[kGroups];
#pragma unroll
                        for (int gi = 0; gi < kGroups; gi++) {
                            sp[gi] = sm.span[kind][gi * kRowsPer + rsub];
                            mt[gi] = sm.meta[kind][gi * kRowsPer + rsub];
                        }
#pragma unroll
                        for (int gi = 0; gi < kGroups; gi++)
                            val[gi] = sm.ring[kind][gi * kRowsPer + rsub][(sp[gi].x + e) & (kTlRing - 1)];
#pragma unroll
                        for (int gi = 0; gi < kGroups; gi++) {
                            const int j = sp[gi].x + e;
                            if (j < sp[gi].y) {
                                const int64_t t0 = double_to_i64(val[gi]);
                                out.start[mt[gi].base + j] = t0;
                                out.end[mt[gi].base + j] = t0 + mt[gi].dur;
                            }
                        }
                    }
                    if (upF > fF) fF = upF;
                    if (upB > fB) fB = upB;
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                }
            }
        }
        (void)kmask; (void)kmask2;

        // data-parallel modelling: window of the gradient all-reduce events on this device
        if (act && dp > 1 && r.G > 0 && sched != 2) {
            const int64_t endB = double_to_i64(own);
            if (cl.bucket <= 0) {
                out.ar_start[q * kMaxPP + s] = endB;
                out.ar_end[q * kMaxPP + s] = endB + allreduce_ns(cl, dp, r.G);
            } else {
                const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
                const int64_t startB = endB - Bd_i;
                const int64_t tot_hi = ws.pbc[vr + hi] + ws.pba[rr + hi];
                const int64_t ar_cap = allreduce_ns(cl, dp, cl.bucket);
                int64_t acc = 0, t = 0, first = -1;
                for (int l = hi - 1; l >= lo; l--) {
                    const int64_t ready = startB + (tot_hi - (ws.pbc[vr + l] + ws.pba[rr + l]));
                    acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
                    const int64_t kb = (int64_t)udiv64((uint64_t)acc, (uint64_t)cl.bucket);
                    if (kb > 0) {
                        const int64_t b0 = t > ready ? t : ready;
                        if (first < 0) first = b0;
                        t = b0 + kb * ar_cap;
                        acc -= kb * cl.bucket;
                    }
                    if (l == lo && acc > 0) {
                        const int64_t b0 = t > ready ? t : ready;
                        if (first < 0) first = b0;
                        t = b0 + allreduce_ns(cl, dp, acc);
                    }
                }
                out.ar_start[q * kMaxPP + s] = first;
                out.ar_end[q * kMaxPP + s] = t;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the staging area is reused by the next item
    }
}

// Bubble analysis of a dumped timeline (Sec. 3.2 lists bubble analysis among the timeline's uses;
// Sec. 5: per-stage, per-micro-batch timestamps let a user locate the bubbles): the idle time of
// the device in front of every stage-task = start of the task - end of the task the device ran
// before it (0, the start of the iteration, for its first task).  The predecessor in device order
// follows from the schedule:
//   GPipe   F(s,j) after F(s,j-1);  B(s,0) after F(s,m-1);  B(s,j) after B(s,j-1)
//   Dapple  with w = min(pp-1-s, m) warm-up forwards:
//           F(s,j) after F(s,j-1) for j <= w, after B(s,j-w-1) for j > w;
//           B(s,j) after F(s,w+j) for j < m-w, else after B(s,j-1) (after F(s,m-1) if j = 0)
//   interleaved  the same order over slots; entries [kind][virtual stage][micro-batch]
//   explicit     the order of the device's list; entries of tasks that are not listed stay untouched
// One workgroup per selected candidate; entries in the layout of the dump, [kind][stage][micro-batch].
__global__ __launch_bounds__(256) void k_bubbles(CandDev ca, const int32_t* __restrict__ status, int64_t C, int64_t n,
                                                 const int64_t* __restrict__ sel, const int64_t* __restrict__ task_off,
                                                 const int64_t* __restrict__ start, const int64_t* __restrict__ end,
                                                 int64_t* __restrict__ idle) {
    const int64_t q = blockIdx.x;
    if (q >= n) return;
    const int64_t c = sel[q];
    if (c < 0 || c >= C || status[c] != 0) return;
    const int pp = ca.pp[c], m = ca.m[c], sched = ca.schedule[c];
    const int64_t off = task_off[q];
    if (sched == 4) {
        // Explicit schedule: the lists are the device order; thread d walks the list of device d.
        if (!ca.chunks || !ca.schedule_off || !ca.schedule_words) return;
        const int32_t* w = ca.schedule_words + ca.schedule_off[ca.chunks[c]];     // checked when the candidate got status OK
        const int S = w[1];
        const int32_t* dev_off = w + 5;
        const int32_t* tasks = dev_off + pp + 1 + 3 * S;
        if ((int)threadIdx.x < pp) {
            int64_t before = 0;
            for (int i = dev_off[threadIdx.x]; i < dev_off[threadIdx.x + 1]; i++) {
                const uint32_t x = (uint32_t)tasks[i];
                const int64_t e = off + ((int64_t)(x >> 31) * S + ((x >> 16) & 0x7fff)) * m + (x & 0xffff);
                idle[e] = start[e] - before;
                before = end[e];
            }
        }
        return;
    }
    if (sched > 4) return;
    if (sched == 3) {
        // Interleaved: device d = k mod pp runs slots, not micro-batches, in the Dapple order with
        // W warm-up forwards.  Slot i of a direction <-> (chunk, micro-batch) and slot <-> position
        // in the device's list are closed forms, so is the task one position earlier.
        if (!ca.chunks) return;
        const int vch = ca.chunks[c];
        const int S = pp * vch, group = pp * vch;
        const int64_t ns = (int64_t)m * vch, per = (int64_t)S * m;
        for (int64_t t = threadIdx.x; t < 2 * per; t += blockDim.x) {
            const int kind = t >= per ? 1 : 0;
            const int64_t r = t - kind * per;
            const int k = (int)(r / m), j = (int)(r - (int64_t)k * m);
            const int d = k % pp, cch = k / pp;
            int64_t W = 2ll * (pp - d - 1) + (int64_t)(vch - 1) * pp;
            if (W > ns) W = ns;
            const int64_t i = (int64_t)(j / pp) * group + (kind == 0 ? cch : vch - 1 - cch) * pp + j % pp;
            const int64_t pos = kind == 0 ? (i < W ? i : W + 2 * (i - W)) : (i < ns - W ? W + 2 * i + 1 : ns + i);
            int64_t before = 0;
            if (pos > 0) {
                const int64_t p = pos - 1;
                int pk;
                int64_t pi;
                if (p < W) { pk = 0; pi = p; }
                else if (p < W + 2 * (ns - W)) { const int64_t x = p - W; pk = (int)(x & 1); pi = pk ? x / 2 : W + x / 2; }
                else { pk = 1; pi = p - ns; }
                const int w = (int)(pi % group), cc = w / pp;
                const int64_t pj = (pi / group) * pp + w % pp;
                const int kk = (pk == 0 ? cc : vch - 1 - cc) * pp + d;
                before = end[off + ((int64_t)pk * S + kk) * m + pj];
            }
            idle[off + t] = start[off + t] - before;
        }
        return;
    }
    const int per_kind = pp * m;                          // <= 64 * 65536
    for (int t = threadIdx.x; t < 2 * per_kind; t += blockDim.x) {
        const int kind = t >= per_kind ? 1 : 0;
        const int r = t - kind * per_kind;
        const int s = r / m, j = r - s * m;
        int pk = -1, pj = 0;                              // predecessor (kind, micro-batch); pk < 0: none
        if (sched == 0) {
            if (j > 0) { pk = kind; pj = j - 1; }
            else if (kind == 1) { pk = 0; pj = m - 1; }
        } else {
            int w = pp - 1 - s; if (w > m) w = m;
            if (kind == 0) {
                if (j > w) { pk = 1; pj = j - w - 1; }
                else if (j > 0) { pk = 0; pj = j - 1; }
            } else {
                if (j < m - w) { pk = 0; pj = w + j; }
                else if (j > 0) { pk = 1; pj = j - 1; }
                else { pk = 0; pj = m - 1; }
            }
        }
        const int64_t before = pk < 0 ? 0 : end[off + ((int64_t)pk * pp + s) * m + pj];
        idle[off + t] = start[off + t] - before;
    }
}

}  // namespace distsim
