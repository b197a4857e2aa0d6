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

// Start times wait in LDS, per (kind, lane), until a 64-byte aligned run of their row of the output
// is complete: a ring that takes what the last flush left behind (fewer than kTlRun entries) plus
// the entries of the kTlRun levels up to the next flush (at most one task of a kind per level).
constexpr int kTlRun = 8;                // entries per aligned run (64 bytes) = levels between two flushes
constexpr int kTlRing = 2 * kTlRun;      // ring capacity per (kind, lane)
constexpr int kTlRowPad = kTlRing + 2;   // padded: the rows of neighbouring lanes start in different LDS banks, every row 16-byte aligned

// Per-wavefront staging area.
struct TlRowMeta { int64_t at, dur_cnt; };   // index in start / end of the first entry to write; task duration (below 2^53) | entries to write << 56
struct TlStage {
    alignas(16) double buf[2][kWave][kTlRowPad];     // [kind][lane][index of the entry in the output modulo kTlRing]
    TlRowMeta meta[2][kWave];
};

// Width class of selection entry q for the level-sweep dump (0: 64 lanes ... 6: one lane), -1 when the
// entry gets no dump from k_timeline: index outside the list, candidate not OK, or a schedule that
// has a dump kernel of its own (GPipe: k_timeline_gpipe; interleaved and explicit schedules).
__device__ __forceinline__ int timeline_class(const CandDev& ca, const int32_t* __restrict__ status, int64_t C, int64_t c) {
    if (c < 0 || c >= C || status[c] != 0 || ca.schedule[c] >= 3 || ca.schedule[c] == 0) return -1;
    const int pp = ca.pp[c];
    int sh = 0;
    while ((1 << sh) < pp) sh++;
    return 6 - sh;
}

// Packing of the selection into wave-items, over the whole selection: a counting sort by width
// class (two passes over the selection), so that the candidates of few stages share wavefronts
// whatever their place in the selection, and every item becomes a wavefront of its own.  Counters:
// cnt[0..6] entries per class, cnt[8..14] the scatter pass's cursors.
constexpr int kTlCounters = 16;
__global__ __launch_bounds__(64) void k_timeline_clear(int32_t* __restrict__ cnt) {
    if (threadIdx.x < kTlCounters) cnt[threadIdx.x] = 0;
}

// PASS 0: counts the entries of every class and sets all all-reduce windows of the selection to
// "none".  PASS 1: hands every entry its place among the entries of its class (a block adds its
// own counts to the cursors once per class) and writes the entry's number there.
template <int PASS>
__global__ __launch_bounds__(256) void k_timeline_pack(CandDev ca, const int32_t* __restrict__ status, int64_t C, int64_t n,
                                                       const int64_t* __restrict__ sel, int32_t* __restrict__ cnt,
                                                       int32_t* __restrict__ sorted, int64_t* __restrict__ ar_start,
                                                       int64_t* __restrict__ ar_end) {
    __shared__ int32_t hist[kClasses], base[kClasses];
    if (threadIdx.x < kClasses) hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int k = q < n ? timeline_class(ca, status, C, sel[q]) : -1;
    int rank = 0;
    if (k >= 0) rank = atomicAdd(&hist[k], 1);
    if (PASS == 0) {
        const int64_t q_first = (int64_t)blockIdx.x * blockDim.x;
        for (int i = threadIdx.x; i < (int)blockDim.x * kMaxPP; i += blockDim.x) {
            const int64_t e = q_first * kMaxPP + i;
            if (e < n * kMaxPP) { ar_start[e] = -1; ar_end[e] = -1; }
        }
    }
    __syncthreads();
    if (threadIdx.x < kClasses && hist[threadIdx.x] > 0)
        base[threadIdx.x] = atomicAdd(&cnt[(PASS == 0 ? 0 : 8) + threadIdx.x], hist[threadIdx.x]);
    if (PASS == 0) return;
    __syncthreads();
    if (k >= 0) {
        int start = 0;                                   // entries of the wider classes come first
        for (int i = 0; i < k; i++) start += cnt[i];
        sorted[start + base[k] + rank] = (int32_t)q;
    }
}

// Data-parallel modelling for the dump: window of the gradient all-reduce events on the device of
// stage s (entry q of the selection), which has dp > 1 replicas and G > 0 gradient bytes.  endB: end
// of the stage's last backward, Bd_i: its duration.
__device__ __forceinline__ void allreduce_window(const ClusterDev& cl, const Workspace& ws, int L, int v, int pp, int dp,
                                                 int lo, int hi, int64_t G, int64_t endB, int64_t Bd_i,
                                                 const TimelineOut& out, int64_t q, int s) {
    if (cl.bucket <= 0) {
        out.ar_start[q * kMaxPP + s] = endB;
        out.ar_end[q * kMaxPP + s] = endB + allreduce_ns(cl, dp, G);
        return;
    }
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

// One wavefront per wave-item of the packed selection (64 >> k entries of class k, 1 << (6 - k)
// lanes each), widest class -- the longest sweeps -- first.
// The sweep is the level sweep of kernels_simulate.hpp (same level functions, bit patterns and
// task step) with one addition: after each step the lanes that ran a task put its start time
// into their row of the staging area.  A stage's tasks of one kind come in micro-batch order and
// their entries are consecutive in the output ([kind][stage][micro-batch]).  Every kTlRun levels the
// wavefront writes out, per row, the entries up to the last 64-byte boundary of the output arrays
// (the rest waits for the next flush; the last flush writes everything), with the lanes regrouped:
// four neighbouring lanes take one row, two entries each, so that one store instruction writes 16
// rows and the four lanes of a row write one whole aligned 64-byte run (one full-width request to
// memory instead of one per lane); end = start + the row's task duration.  The staging area
// belongs to one wavefront, whose LDS instructions execute in order: between its writes and the
// reads by other lanes only the compiler has to be kept from reordering (wavefront-scope fences).
__global__ __launch_bounds__(kWave) void k_timeline(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                    const int32_t* __restrict__ status, int64_t C, int64_t n,
                                                    const int32_t* __restrict__ cnt, const int32_t* __restrict__ sorted,
                                                    TimelineOut out) {
    __shared__ TlStage stage_mem;
    const int lane = lane_id();
    const int L = co.L;
    // class and item ranges from the counts (wave-uniform)
    int cls_start[kClasses + 1], item_start[kClasses + 1];
    cls_start[0] = 0; item_start[0] = 0;
#pragma unroll
    for (int kk = 0; kk < kClasses; kk++) {
        const int c_k = cnt[kk];
        cls_start[kk + 1] = cls_start[kk] + c_k;
        item_start[kk + 1] = item_start[kk] + ((c_k + (1 << kk) - 1) >> kk);
    }
    const int total_items = item_start[kClasses];
    TlStage& sm = stage_mem;
    const double ninf = -__builtin_huge_val();
    for (int w = blockIdx.x; w < total_items; w += gridDim.x) {
        int k = 0, first_item = 0, first_entry = 0, class_entries = 0;
#pragma unroll
        for (int kk = 0; kk < kClasses; kk++)
            if (w >= item_start[kk]) { k = kk; first_item = item_start[kk]; first_entry = cls_start[kk]; class_entries = cls_start[kk + 1] - cls_start[kk]; }
        const int sh = 6 - k, width = 1 << sh;
        const int g = lane >> sh, s = lane & (width - 1);
        const int slot = ((w - first_item) << k) + g;             // position inside the class
        const bool have = slot < class_entries;
        const int64_t q = have ? sorted[first_entry + slot] : 0;
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

        // level windows of this lane on x = level - s (see kernels_simulate.hpp)
        const LevelWindows lw(m, pp, s);
        const int f1hi = lw.f1hi, f2lo = lw.f2lo, f2hi = lw.f2hi, blo = lw.blo, bhi = lw.bhi;
        const int nlev = wave_max_i32(act ? 2 * (m + pp - 1) : 0);
        double own = 0.0;
        double linkF = 0.0, linkB = 0.0;                      // p2p_blocking = 2: arrival of the lane's latest sends
        const double sendF = (double)r.PF, sendB = (double)r.PB;
        const bool hasL = act && s > 0, hasR = act && s + 1 < pp;
        int nF = 0, nB = 0, cF = 0, cB = 0;                   // tasks written out / staged since the last flush, per kind
        const int ringF = (int)baseF & (kTlRing - 1), ringB = (int)baseB & (kTlRing - 1);      // ring slot of the row's first entry
        uint64_t kmask = 0, kmask2 = 0;
        for (int l0 = 0; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;
            uint32_t PFb = level_bits(-x0, f1hi - x0) | (level_bits(f2lo - x0, f2hi - x0) & even_x);
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;
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
                // an entry's ring slot is its index in the output modulo the ring: runs that are aligned
                // in the output are aligned in the ring too
                if (ranF) { sm.buf[0][lane][(ringF + nF + cF) & (kTlRing - 1)] = tF; cF++; }
                if (ranB) { sm.buf[1][lane][(ringB + nB + cB) & (kTlRing - 1)] = tB; cB++; }
                const bool last = l0 + kk == nlev - 1;
                if ((kk & (kTlRun - 1)) != kTlRun - 1 && !last) continue;
                // flush: per kind and row the staged entries up to the last 64-byte boundary of the
                // output (all of them in the last flush, which may take two rounds)
                // every time of the item so far is at most some lane's `own`: below 2^52 they convert with one addition
                const bool small = __builtin_amdgcn_ballot_w64(own >= 4503599627370496.0) == 0;
                for (int kind = 0; kind < 2; kind++)
                for (int round = 0; round < (last ? 2 : 1); round++) {
                    const int64_t at = kind ? baseB + nB : baseF + nF;
                    const int staged = kind ? cB : cF;
                    int wr = last ? staged : staged - (((int)at + staged) & (kTlRun - 1));
                    wr = wr < 0 ? 0 : (wr > kTlRun ? kTlRun : wr);
                    if (__builtin_amdgcn_ballot_w64(wr > 0) == 0) continue;
                    // whole aligned runs only (the usual flush): pairs of entries are 16-byte aligned in the ring and in the output
                    const bool whole = __builtin_amdgcn_ballot_w64(wr > 0 && (wr != kTlRun || ((int)at & (kTlRun - 1)) != 0)) == 0;
                    sm.meta[kind][lane] = TlRowMeta{at, (kind ? Bd_i : Fd_i) | ((int64_t)wr << 56)};
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    constexpr int kLanesPerRow = kTlRun / 2, kRowsPer = kWave / kLanesPerRow;      // 4 lanes x 2 entries; 16 rows per store
                    constexpr int kStores = kWave / kRowsPer;
                    const int rsub = lane / kLanesPerRow, e = 2 * (lane % kLanesPerRow);
                    // all LDS reads of the four stores first, then the stores
                    TlRowMeta mt[kStores];
                    double v0[kStores], v1[kStores];
#pragma unroll
                    for (int gi = 0; gi < kStores; gi++) mt[gi] = sm.meta[kind][gi * kRowsPer + rsub];
                    if (whole && small) {
#pragma unroll
                        for (int gi = 0; gi < kStores; gi++) {
                            const int r = gi * kRowsPer + rsub, sl = ((int)mt[gi].at + e) & (kTlRing - 1);      // even
                            const double2 v = *reinterpret_cast<const double2*>(&sm.buf[kind][r][sl]);
                            v0[gi] = v.x; v1[gi] = v.y;
                        }
#pragma unroll
                        for (int gi = 0; gi < kStores; gi++) {
                            if ((mt[gi].dur_cnt >> 56) != 0) {
                                const int64_t dur = mt[gi].dur_cnt & (((int64_t)1 << 56) - 1);
                                const int64_t a = small_double_to_i64(v0[gi]), b = small_double_to_i64(v1[gi]);
                                const int64_t idx = mt[gi].at + e;
                                // written once and not read again by this kernel: streaming stores
                                typedef long long i64x2 __attribute__((ext_vector_type(2)));
                                __builtin_nontemporal_store(i64x2{a, b}, reinterpret_cast<i64x2*>(out.start + idx));
                                __builtin_nontemporal_store(i64x2{a + dur, b + dur}, reinterpret_cast<i64x2*>(out.end + idx));
                            }
                        }
                    } else {
#pragma unroll
                        for (int gi = 0; gi < kStores; gi++) {
                            const int r = gi * kRowsPer + rsub, sl = (int)mt[gi].at + e;
                            v0[gi] = sm.buf[kind][r][sl & (kTlRing - 1)];
                            v1[gi] = sm.buf[kind][r][(sl + 1) & (kTlRing - 1)];
                        }
#pragma unroll
                        for (int gi = 0; gi < kStores; gi++) {
                            const int n_row = (int)(mt[gi].dur_cnt >> 56);
                            const int64_t dur = mt[gi].dur_cnt & (((int64_t)1 << 56) - 1);
                            if (e < n_row) {
                                const int64_t a = double_to_i64(v0[gi]), b = double_to_i64(v1[gi]);
                                const int64_t idx = mt[gi].at + e;
                                if (e + 1 < n_row) {
                                    *reinterpret_cast<longlong2*>(out.start + idx) = longlong2{a, b};
                                    *reinterpret_cast<longlong2*>(out.end + idx) = longlong2{a + dur, b + dur};
                                } else {
                                    out.start[idx] = a;
                                    out.end[idx] = a + dur;
                                }
                            }
                        }
                    }
                    if (kind) { nB += wr; cB -= wr; } else { nF += wr; cF -= wr; }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                }
            }
        }
        (void)kmask; (void)kmask2;

        if (act && dp > 1 && r.G > 0 && sched != 2)
            allreduce_window(cl, ws, L, v, pp, dp, lo, hi, r.G, double_to_i64(own), Bd_i, out, q, s);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the staging area is reused by the next item
    }
}

// The GPipe candidates of the selection, without a sweep: every task's end has the closed form
// that gpipe_finish (kernels_simulate.hpp) derives,
//   end F(s, j) = sum_{i<=s} (F_i + pf_i) + j max_{i<=s} F_i
//   end B(s, j) = end F(pp-1, m-1) + sum_{i>=s} (B_i + pb_i) + j max_{i>=s} B_i
// and start = end - duration.  One workgroup per selected candidate: lane s of its first wavefront
// forms the four scans of stage s and leaves (end of the first task, step per micro-batch,
// duration) of its two rows in LDS; then all threads write the candidate's block entry by entry,
// consecutive threads consecutive entries, every wavefront 512 contiguous bytes of each array per
// store instruction.  With p2p_blocking = 2 (sends queue on their links) a link is one more machine
// of the flow shop and its transfer time enters the two maxima.
constexpr int kTlGpipeBlock = 256;
struct alignas(16) TlGpipeRow { double end0, step, dur, spare; };
__global__ __launch_bounds__(kTlGpipeBlock) void k_timeline_gpipe(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                                  const int32_t* __restrict__ status, int64_t C, int64_t n,
                                                                  TimelineOut out) {
    __shared__ TlGpipeRow tab[2 * kWave];
    __shared__ int verdict;                 // 0: no entries for this candidate, 1: times below 2^52, 2: above
    const int lane = lane_id(), s = lane;
    const bool first_wave = threadIdx.x < kWave;
    const int L = co.L;
    // q, hence everything that decides whether an entry of the selection is taken, is the same in
    // all threads of the workgroup
    for (int64_t q = blockIdx.x; q < n; q += gridDim.x) {
        const int64_t c = out.sel[q];
        if (c < 0 || c >= C) continue;
        if (status[c] != 0 || ca.schedule[c] != 0) continue;
        const int pp = __builtin_amdgcn_readfirstlane(ca.pp[c]), m = __builtin_amdgcn_readfirstlane(ca.m[c]);
        if (first_wave) {
            const int dp = ca.dp[c], tp = ca.tp[c];
            const int64_t poff = ca.part_off[c];
            int v = 0;
            for (int i = co.V - 1; i >= 0; i--) if (co.variant_tp[i] == tp) v = i;
            const bool in = s < pp;
            int lo = 0, hi = 0;
            if (in) {
                if (poff >= 0) { lo = ca.part_pool[poff + s]; hi = ca.part_pool[poff + s + 1]; }
                else { lo = uniform_bound(s, L, pp); hi = uniform_bound((s + 1), L, pp); }
            }
            StageRow r;
            // a candidate whose partition or range check fails gets no entries
            const bool ok = stage_row(cl, ws, L, kWave, s, pp, v, m, dp, tp, lo, hi, r) == 0;
            const int64_t pf_task = cl.blocking == 1 ? r.PF : 0, pb_task = cl.blocking == 1 ? r.PB : 0;
            const int64_t Fd_i = r.FC + r.FA + pf_task, Bd_i = r.BC + r.BA + pb_task;
            const double Fd = (double)Fd_i, Bd = (double)Bd_i;              // zero in lanes without a stage
            // latency of the edge into the stage (the neighbour's outgoing event), zero without one
            double pfL = from_prev_lane((double)(r.PF - pf_task)), pbR = from_next_lane((double)(r.PB - pb_task));
            if (!(in && s > 0)) pfL = 0.0;
            if (!(in && s + 1 < pp)) pbR = 0.0;
            // prefix sum and maximum over the stages up to s, suffix sum and maximum over those from s on
            double A = Fd + pfL, MF = Fd, T = Bd + pbR, MB = Bd;
            if (cl.blocking == 2) { MF = max_f64(Fd, pfL); MB = max_f64(Bd, pbR); }
            for (int d = 1; d < kWave; d <<= 1) {
                const bool up = lane >= d, dn = lane + d < kWave;
                const int au = (up ? lane - d : lane) * 4, ad = (dn ? lane + d : lane) * 4;
                const double a = from_lanes(A, au), f = from_lanes(MF, au), t = from_lanes(T, ad), b = from_lanes(MB, ad);
                A += up ? a : 0.0;
                MF = max_f64(MF, f);
                T += dn ? t : 0.0;
                MB = max_f64(MB, b);
            }
            const double mm1 = (double)(m - 1);
            const double R = readlane_f64(A, pp - 1) + mm1 * readlane_f64(MF, pp - 1);   // end of the last stage's last forward
            if (in) {
                tab[s] = TlGpipeRow{A, MF, Fd, 0.0};
                tab[kWave + s] = TlGpipeRow{R + T, MB, Bd, 0.0};
            }
            // the last task of all ends at stage 0: below 2^52 every time converts with one addition
            const bool small = R + readlane_f64(T, 0) + mm1 * readlane_f64(MB, 0) < 4503599627370496.0;
            if (lane == 0) verdict = ok ? (small ? 1 : 2) : 0;
            if (ok && in && dp > 1 && r.G > 0)
                allreduce_window(cl, ws, L, v, pp, dp, lo, hi, r.G, double_to_i64(R + T + mm1 * MB), Bd_i, out, q, s);
        }
        __syncthreads();
        const int vd = verdict;
        if (vd != 0) {
            const bool small = vd == 1;
            const int64_t off = out.task_off[q];
            const int total = 2 * pp * m;                       // [kind][stage][micro-batch], row = kind * pp + stage
            // a step of one workgroup's worth of entries, in rows and micro-batches
            const int qs = kTlGpipeBlock / m, rs = kTlGpipeBlock - qs * m;
            // the 64 entries of a store instruction start at a 128-byte boundary of the output: whole
            // lines but for the two ends of the block.  A thread whose first entry would lie in front
            // of the block starts one turn later, with the row and micro-batch of that later entry.
            const int skew = (int)((reinterpret_cast<uintptr_t>(out.start + off) >> 3) & 15);
            int e = (int)threadIdx.x - skew;
            const int e_first = e < 0 ? e + kTlGpipeBlock : e;
            int row = e_first / m, j = e_first - row * m;
            for (int base = -skew; base < total; base += kTlGpipeBlock, e += kTlGpipeBlock) {
                if (e < 0 || e >= total) continue;
                const TlGpipeRow t = tab[row < pp ? row : row + (kWave - pp)];
                const double en = t.end0 + (double)j * t.step, st = en - t.dur;
                const int64_t a = small ? small_double_to_i64(st) : double_to_i64(st);
                const int64_t b = small ? small_double_to_i64(en) : double_to_i64(en);
                // written once and not read again by this kernel: streaming stores
                __builtin_nontemporal_store(a, out.start + off + e);
                __builtin_nontemporal_store(b, out.end + off + e);
                j += rs; row += qs;
                if (j >= m) { j -= m; row++; }
            }
        }
        __syncthreads();                    // the rows are reused by the next entry
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
    // the task in front of task t on its device: index into start / end, -1 = none
    auto predecessor = [&](int t) -> int64_t {
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
        return pk < 0 ? -1 : off + ((int64_t)pk * pp + s) * m + pj;
    };
    // four tasks per thread and turn, all their loads before the first store: the kernel waits for
    // memory, not for arithmetic
    constexpr int kPer = 4;
    const int total = 2 * per_kind;
    for (int t0 = threadIdx.x; t0 < total; t0 += kPer * blockDim.x) {
        int64_t st[kPer], before[kPer];
#pragma unroll
        for (int u = 0; u < kPer; u++) {
            const int t = t0 + u * blockDim.x;
            const int64_t p = t < total ? predecessor(t) : -1;
            st[u] = t < total ? start[off + t] : 0;
            before[u] = p >= 0 ? end[p] : 0;
        }
#pragma unroll
        for (int u = 0; u < kPer; u++) {
            const int t = t0 + u * blockDim.x;
            if (t < total) idle[off + t] = st[u] - before[u];
        }
    }
}

}  // namespace distsim
