// Interleaved one-forward-one-backward schedule: every device holds several model chunks, so a
// device's tasks belong to several virtual stages and the producer of a task is no longer "the
// neighbour's latest task".  A wavefront is cut into groups of R lanes, one candidate per group,
// lane = device.  Each lane walks its own task list (closed forms of the slot numbers, see
// distsim.h) and keeps the end times of its latest forward and backward slots in short LDS rings.
// A round is a forward step and a backward step: in the forward step the lanes whose next task is
// a forward run it if the producing slot on the neighbouring device (the device before for
// forwards, after for backwards) has been run, reading its end time from that device's ring; the
// backward step does the same for the lanes whose next task is then a backward, so a device in
// the steady phase runs both tasks of a pair in one round, each in code that knows its direction.
// The edge from the last device back to the first joins slots one chunk (pp slots) apart and has
// a longer ring of its own.  Rounds repeat until every list of the wavefront is done; a round in
// which no lane can run ends the loop (it cannot happen for a valid schedule) and the candidates
// still unfinished are reported invalid.  Same arithmetic as the level sweep: fp64 values that
// are integers below 2^53.
#pragma once
#include <cstddef>
#include <type_traits>

#include "kernels_simulate.hpp"

namespace distsim {

// LDS of one wavefront, which holds 64 / R candidates of at most R devices each (R a power of
// two, 2 to 64).  Two kinds of ring hold task ends, both per direction: one of kDepth slots per
// device, read by the next device of the direction at the same slot number, and one of R slots
// per candidate, written by the direction's last device and read by its first device pp slots
// later.  The steps do not depend on the durations, so running them on the CPU settles the
// depths (every pp, every chunk count with pp * chunks <= 64, micro-batch counts up to 8 pp): a
// device leads the next one by at most 2 slots, the last device leads the first by up to pp / 2
// slots on top of the pp between them, and with these depths no schedule waits for a slot to
// become free (2 m chunks + about 2 pp steps in all).  A task that would overwrite a slot not
// yet read waits, so a ring that were too small could stall a candidate but never give a wrong
// time.  The table of virtual stages is shared by the wavefront's candidates: each takes pp *
// chunks entries, and candidates that do not fit wait for a further pass (none do with up to
// 128 / (64 / R) virtual stages each, e.g. two chunks per device).
struct VirtStage {                              // one virtual stage: task durations, latencies of the incoming edges
    double dur_f, lat_f, dur_b, lat_b;
};
struct VirtLds {
    static constexpr int kDepth = 2, kStages = 2 * kWave;
    // first index of the rings and counters: direction, 0 = forward, 1 = backward
    double ring[2][kDepth][kWave];              // by slot modulo kDepth and lane: what the next device reads
    double wrap[2][kWave];                      // R slots per candidate, slot modulo R: the same from the direction's last device
    alignas(32) VirtStage st[kStages];          // the candidates' virtual stages, one candidate after the other
    int32_t done[2][kWave];                     // by lane: slots run
};

// What a lane needs for its tasks of one direction.  Places in LDS are byte offsets from the start
// of the wavefront's VirtLds.
struct VirtDir {
    int a_done_src, a_done_cons, a_done_own;    // slot counters of the producing device, of the consuming device, of this one
    int p_base, p_off, p_mask, p_sh;            // the producer's end of slot i: p_base + (((i - p_off) & p_mask) << p_sh)
    int m_base, m_mask, m_sh;                   // where this lane's end of slot i goes: m_base + ((i & m_mask) << m_sh)
    int g_min, g_off;                           // slot i may go there if i < g_min or the consumer has run more than i - g_off slots
    int k_first, k_last;                        // virtual stages without a producer / without a consumer (direction's ends)
    int k_start, k_step;                        // stage of the first chunk in this direction's order, step to the next chunk
};
// The slot a lane is at in one direction: slot i = round of pp * chunks slots (first micro-batch
// j0), chunk position cp in the direction's order, place r in the chunk; k = virtual stage.
struct VirtPos {
    int i, r, cp, j0, k;
};

// What one candidate needs from its descriptor (or, for the dump, from the candidate arrays); the
// lanes of a group hold the same values.  pp == 0: the group has no candidate.
struct VirtCand {
    int pp, v, m, dp, tp, vch;
    int st0;             // first entry of the candidate in the table of virtual stages
    int64_t poff, c;
};

// Where the dump of one candidate goes (the simulation proper passes none).
struct VirtDump {
    int64_t* start;      // [2][pp * vch][m]
    int64_t* end;
    int64_t* ar_start;   // [kMaxPP] by device
    int64_t* ar_end;
};

// The candidates of one wavefront, one per group of R lanes.  DUMP = false: writes status
// / batch time / busy sums.  DUMP = true: the candidates are known to be OK; writes every task's
// start and end and the all-reduce windows, and none of the simulation's outputs.
template <bool DUMP, int R>
__device__ __forceinline__ void virtual_groups(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                               const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                               const VirtCand& vc, const VirtDump& dump, VirtLds& sm) {
    static_assert(R >= 2 && R <= kWave && (R & (R - 1)) == 0, "group sizes are powers of two from 2 to 64");
    constexpr int D = VirtLds::kDepth;
    using Lds = VirtLds;
    VirtStage* const st = sm.st + vc.st0;                         // this candidate's virtual stages
    const int lane = threadIdx.x;
    const int g = lane / R, d = lane % R, g0 = g * R;            // group, device, first lane of the group
    const int L = co.L;
    const int pp = vc.pp, v = vc.v, m = vc.m, dp = vc.dp, tp = vc.tp, vch = vc.vch;
    const int64_t c = vc.c;
    const int S = pp * vch;
    bool act = d < pp;                                           // pp == 0: nothing to do in this group
    const int64_t tpdp = (int64_t)tp * dp;
    auto node_of = [&](int dev) -> int64_t {
        return tpdp >= cl.gpus_per_node ? dev : (int64_t)node_of_position(cl, dev, (int)tpdp);
    };
    const int64_t* row = ws.comb + (size_t)((v * kMaxPP + (pp > 0 ? pp - 1 : 0)) * (L + 1)) * kCombWords;

    // composed events of this device's chunks
    int bad = 0;
    int64_t comp = 0, comm = 0, G = 0, share = 0;
    if (act) {
        const int64_t my_node = node_of(d), next_node = node_of((d + 1) % pp), prev_node = node_of((d + pp - 1) % pp);
        for (int cch = 0; cch < vch; cch++) {
            const int k = cch * pp + d;
            int lo, hi;
            if (vc.poff >= 0) { lo = ca.part_pool[vc.poff + k]; hi = ca.part_pool[vc.poff + k + 1]; }
            else { lo = uniform_bound(k, L, S); hi = uniform_bound((k + 1), L, S); }
            if (hi <= lo || hi > L || (k == 0 && lo != 0) || (k == S - 1 && hi != L)) { bad = 1; break; }
            const int64_t* eh = row + hi * kCombWords;
            const int64_t* el = row + lo * kCombWords;
            const int64_t FT = eh[0] - el[0], BT = eh[1] - el[1], CP = eh[2] - el[2];
            const int64_t PF = k + 1 < S ? eh[4 + (my_node != next_node ? 1 : 0)] : 0;
            const int64_t PB = k > 0 ? el[4 + (my_node != prev_node ? 1 : 0)] : 0;
            G += eh[3] - el[3];
            comp += CP;
            comm += FT + BT - CP + PF + PB;
            share += FT + BT + PF + PB;
            const int64_t pf_task = cl.blocking == 1 ? PF : 0, pb_task = cl.blocking == 1 ? PB : 0;
            VirtStage vs;
            vs.dur_f = (double)(FT + pf_task);
            vs.dur_b = (double)(BT + pb_task);
            // A boundary's p2p event is the same in both directions, so the latency of the edge into
            // this stage equals the stage's own transfer across that boundary the other way: the
            // forward edge comes over the boundary that the backward send crosses, and vice versa.
            vs.lat_f = (double)(PB - pb_task);
            vs.lat_b = (double)(PF - pf_task);
            st[k] = vs;
        }
    }
    const bool gbad = group_any(bad != 0, R);
    const bool range = stage_out_of_range(act && !gbad ? share : 0, m, R);
    if (gbad || range) {
        if (!DUMP && act && d == 0) { ev.status[c] = gbad ? 1 : 2; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        act = false;
    }
    // (a lane reads only its own stages' entries: no barrier is needed for them)

    // the rounds
    // slot numbers fit 32 bits: m <= 2^16 and pp * vch <= 64
    const int n = act ? m * vch : 0;                          // slots per direction
    int W = 2 * (pp - d - 1) + (vch - 1) * pp;                // warm-up forwards
    if (W > n) W = n;
    // Per direction: the producer of a slot is the same slot on the device before (in the
    // direction), or, on the direction's first device, the slot pp earlier on its last device,
    // which sits in the candidate's wrap ring; the consumer of the ring slot that a task
    // overwrites is the device after or, on the direction's last device, the first device (pp
    // slots later).
    char* const lds = reinterpret_cast<char*>(&sm);
    const int dLast = pp > 0 ? pp - 1 : 0;
    auto dir_consts = [&](int dir) {
        const bool fwd = dir == 0;
        const bool first = fwd ? d == 0 : d == dLast, last = fwd ? d == dLast : d == 0;
        const int before = fwd ? (d > 0 ? d - 1 : 0) : (d < dLast ? d + 1 : d);       // clamped: unused at the ends
        const int after = fwd ? (d < dLast ? d + 1 : d) : (d > 0 ? d - 1 : 0);
        const int src = g0 + (first ? (fwd ? dLast : 0) : before), cons = g0 + (last ? (fwd ? 0 : dLast) : after);
        const int ring0 = (int)offsetof(Lds, ring) + dir * D * kWave * 8, wrap0 = (int)offsetof(Lds, wrap) + (dir * kWave + g0) * 8;
        const int done0 = (int)offsetof(Lds, done) + dir * kWave * 4;
        VirtDir dc;
        dc.a_done_src = done0 + src * 4; dc.a_done_cons = done0 + cons * 4; dc.a_done_own = done0 + lane * 4;
        dc.p_base = first ? wrap0 : ring0 + src * 8; dc.p_off = first ? pp : 0;
        dc.p_mask = first ? R - 1 : D - 1; dc.p_sh = first ? 3 : 9;
        dc.m_base = last ? wrap0 : ring0 + lane * 8; dc.m_mask = last ? R - 1 : D - 1; dc.m_sh = last ? 3 : 9;
        dc.g_min = last ? (vch > 1 ? R : INT32_MAX) : D; dc.g_off = last ? R - pp : D;
        dc.k_first = fwd ? 0 : S - 1; dc.k_last = fwd ? S - 1 : 0;
        dc.k_start = fwd ? d : (vch - 1) * pp + d; dc.k_step = fwd ? pp : -pp;
        return dc;
    };
    static_assert(kWave * 8 == 1 << 9, "a ring slot is 64 doubles apart from the next");
    const VirtDir dcF = dir_consts(0), dcB = dir_consts(1);
    VirtPos pF{0, 0, 0, 0, dcF.k_start}, pB{0, 0, 0, 0, dcB.k_start};
    double own = 0.0;
    // p2p_blocking = 2: a link is an ordered pair (sending device, receiving device) and carries one
    // transfer at a time.  A device sends forwards to the device after it and backwards to the one
    // before it (both modulo pp): two queues, which are one and the same for pp <= 2.
    double link_f = 0.0, link_b = 0.0;
    const bool one_queue = pp <= 2;
    if (act) {
        *reinterpret_cast<int32_t*>(lds + dcF.a_done_own) = 0;
        *reinterpret_cast<int32_t*>(lds + dcB.a_done_own) = 0;
    }
    __syncthreads();
    // One step: the lanes in `want` try their next task of the direction.  All LDS reads come
    // before the writes, so what a lane sees does not depend on the order of the lanes.
    auto step = [&](auto dir_tag, auto links_tag, const VirtDir& dc, VirtPos& p, double& link, bool want) -> bool {
        constexpr int dir = decltype(dir_tag)::value;
        constexpr bool LINKS = decltype(links_tag)::value;               // p2p_blocking = 2
        bool ran = false;
        if (want) {
            const int i = p.i, si = i - dc.p_off;
            const int done_src = *reinterpret_cast<const int32_t*>(lds + dc.a_done_src);
            const int done_cons = *reinterpret_cast<const int32_t*>(lds + dc.a_done_cons);
            const double prod_end = *reinterpret_cast<const double*>(lds + dc.p_base + ((si & dc.p_mask) << dc.p_sh));
            const VirtStage* stg = st + p.k;
            const double dur = dir == 0 ? stg->dur_f : stg->dur_b, lat = dir == 0 ? stg->lat_f : stg->lat_b;
            const bool has_prod = p.k != dc.k_first;
            // one wait for the four reads: without this the compiler moves two of them behind the
            // test below and a step waits for LDS twice
            asm volatile("" : : "v"(prod_end), "v"(dur), "v"(lat), "v"(done_src), "v"(done_cons));
            // the producer has run, and the slot this task overwrites in its ring has been read
            // (no short-circuit: all reads are issued before the first wait)
            const bool ok = (!has_prod | (done_src > si)) & ((i < dc.g_min) | (done_cons > i - dc.g_off));
            if (ok) {
                // with queues on the links the producer has stored the transfer's arrival time
                const double arrive = has_prod ? (LINKS ? prod_end : prod_end + lat) : 0.0;
                const double t0 = max_f64(arrive, own);
                own = t0 + dur;
                double seen = own;                                     // what the consuming task reads
                if (LINKS && p.k != dc.k_last) {
                    // the transfer crosses the boundary of the opposite edge into this stage
                    const double send = dir == 0 ? stg->lat_b : stg->lat_f;
                    seen = max_f64(own, link) + send;
                    link = seen;
                }
                *reinterpret_cast<double*>(lds + dc.m_base + ((i & dc.m_mask) << dc.m_sh)) = seen;
                *reinterpret_cast<int32_t*>(lds + dc.a_done_own) = i + 1;
                const int j = p.j0 + p.r;                              // micro-batch of the slot
                // bucketed all-reduce: the chunk's gradients are complete in this task; its duration is
                // not needed again (the chunk has no later backward), so the start time takes its place
                if (dir == 1 && cl.bucket > 0 && j == m - 1) st[p.k].dur_b = t0;
                if (DUMP) {
                    const int64_t e = ((int64_t)dir * S + p.k) * m + j;
                    dump.start[e] = double_to_i64(t0);
                    dump.end[e] = double_to_i64(own);
                }
                p.i = i + 1;
                if (++p.r == pp) {
                    p.r = 0; p.k += dc.k_step;
                    if (++p.cp == vch) { p.cp = 0; p.k = dc.k_start; p.j0 += pp; }
                }
                ran = true;
            }
        }
        return ran;
    };
    const int max_rounds = wave_max_i32(act ? 4 * n + 8 * pp + 64 : 0);
    // The loop exists twice, with and without the queues on the links, so that neither pays for the other.
    auto rounds = [&](auto links_tag) {
        constexpr bool LINKS = decltype(links_tag)::value;
        for (int round = 0; round < max_rounds; round++) {
            // A device's next task is a forward while it has run at most W forwards more than backwards
            // (W of them in the warm-up, then one before every backward) and forwards are left.  A step
            // that no lane wants is skipped by the branch around its body.  (n = 0 in idle lanes.)
            const bool wantF = pF.i < n && pF.i - pB.i <= W;
            bool ran = step(std::integral_constant<int, 0>{}, links_tag, dcF, pF, link_f, wantF);
            if (LINKS && one_queue) link_b = link_f;
            const bool wantB = pB.i < n && !(pF.i < n && pF.i - pB.i <= W);
            ran |= step(std::integral_constant<int, 1>{}, links_tag, dcB, pB, link_b, wantB);
            if (LINKS && one_queue) link_f = link_b;
            if (__builtin_amdgcn_ballot_w64(ran) == 0) break;           // all lists are done, or nothing can run any more
        }
    };
    if (cl.blocking == 2) rounds(std::true_type{});
    else rounds(std::false_type{});
    const int iB = pB.i;
    __syncthreads();
    // a candidate with a list that did not end: its schedule cannot be run
    if (group_any(act && iB < n, R)) {
        if (!DUMP && act && d == 0) { ev.status[c] = 1; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        act = false;
    }

    // data-parallel modelling per device: one trailing all-reduce over the bytes of all its chunks,
    // or, with a bucket size, the device's buckets: the chunks' gradients arrive in the order of
    // their backwards of the last micro-batch (chunk vch - 1 first), layer by layer from a chunk's
    // last layer down, each at the start of that backward + the backward events down to the layer;
    // full buckets are issued at once and queue, the rest goes after the device's last gradient.
    const int64_t endB = double_to_i64(own);
    const bool has_ar = act && dp > 1 && G > 0;
    int64_t AR = 0, ar_first = endB, finish = endB, nar_dev = has_ar ? 1 : 0;       // AR: busy time of the all-reduce events
    if (has_ar && cl.bucket <= 0) {
        AR = allreduce_ns(cl, dp, G);
        finish = endB + AR;
    } else if (has_ar) {
        const int64_t ar_cap = allreduce_ns(cl, dp, cl.bucket);
        int64_t t_free = 0, acc = 0, ready = 0;
        ar_first = -1; nar_dev = 0;
        for (int cch = vch - 1; cch >= 0; cch--) {
            const int k = cch * pp + d;
            int lo, hi;
            if (vc.poff >= 0) { lo = ca.part_pool[vc.poff + k]; hi = ca.part_pool[vc.poff + k + 1]; }
            else { lo = uniform_bound(k, L, S); hi = uniform_bound((k + 1), L, S); }
            const int64_t startB = double_to_i64(st[k].dur_b), tot_hi = row[hi * kCombWords + 1];
            for (int l = hi - 1; l >= lo; l--) {
                ready = startB + (tot_hi - row[l * kCombWords + 1]);
                acc += row[(l + 1) * kCombWords + 3] - row[l * kCombWords + 3];
                const int64_t kb = (int64_t)udiv64_by((uint64_t)acc, (uint64_t)cl.bucket, cl.inv_bucket);
                if (kb > 0) {
                    const int64_t b0 = t_free > ready ? t_free : ready;
                    if (ar_first < 0) ar_first = b0;
                    t_free = b0 + kb * ar_cap;
                    acc -= kb * cl.bucket;
                    AR += kb * ar_cap; nar_dev += kb;
                }
            }
        }
        if (acc > 0) {
            const int64_t b0 = t_free > ready ? t_free : ready, dd = allreduce_ns(cl, dp, acc);
            if (ar_first < 0) ar_first = b0;
            t_free = b0 + dd;
            AR += dd; nar_dev++;
        }
        finish = t_free > endB ? t_free : endB;
        if (DUMP) { dump.ar_start[d] = ar_first; dump.ar_end[d] = t_free; return; }
    }
    if (DUMP) {
        if (has_ar) { dump.ar_start[d] = endB; dump.ar_end[d] = endB + AR; }
        return;
    }
    const int64_t batch = group_max(act ? finish : 0, R);
    const int64_t nar = group_sum(nar_dev, R);
    if (act) {
        const int64_t base = ev.stage_pos[c];
        if (base >= 0) {
            const int64_t cb = (int64_t)m * comp, mb = (int64_t)m * comm + AR;
            out.comp_busy[base + d] = cb;
            out.comm_busy[base + d] = mb;
            if (out.util) out.util[base + d] = batch > 0 ? (double)cb / (double)batch : 0.0;
        }
        if (d == 0) {
            out.batch_ns[c] = batch;
            ev.num_events[c] = 2ll * m * S + 2ll * m * (S - 1) + nar;
        }
    }
}

// One unit of work: the 64 / R consecutive candidates of the visiting order from pos0 on, one per
// group of R lanes.  Neighbours in visiting order have about the same number of micro-batches,
// hence lists of about the same length when their chunk counts agree.
template <int R>
__device__ __forceinline__ void virtual_unit(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                             const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                             int64_t pos0, int64_t pos_end, VirtLds& sm) {
    constexpr int kGroups = kWave / R;
    const int lane = threadIdx.x, g = lane / R;
    // descriptors beyond the valid candidates were never written: the class table bounds them
    Desc ds{};
    if (pos0 + g < pos_end) ds = ws.desc[pos0 + g];
    if (!is_interleaved(ds)) ds.meta = 0;
    const int pp = ds.meta & 0xff, vch = (int)(ds.spare >> 32);
    bool pending = pp != 0;
    // Passes: the pending candidates, in order, for as long as their virtual stages fit the table
    // (the first always does: a candidate has at most 64).
    for (int pass = 0; pass < kGroups && __builtin_amdgcn_ballot_w64(pending) != 0; pass++) {
        int upto = pending && lane % R == 0 ? pp * vch : 0;        // becomes: stages of the pending candidates up to this one
        for (int sh = 1; sh < kWave; sh <<= 1) {
            const int o = __shfl_up(upto, sh, kWave);
            if (lane >= sh) upto += o;
        }
        const bool now = pending && upto <= VirtLds::kStages;
        const VirtCand vc{now ? pp : 0, ds.meta >> 16, ds.m, ds.dp, (int)(uint32_t)ds.spare, vch,
                          now ? upto - pp * vch : 0, ds.poff, ds.cand};
        virtual_groups<false, R>(co, cl, ca, ws, ev, out, vc, VirtDump{}, sm);
        pending = pending && !now;
    }
}

// Class k of the visiting order holds the candidates of 64 >> k lanes (pp <= 64 >> k), so that a
// wavefront takes 1, 2, 4, 8, 16 or 32 of them (the candidates of one device use groups of two
// lanes), and a class keeps its interleaved candidates side by side, longest lists first.  The
// units of all classes are numbered in one sequence, widest class first, and dealt to the blocks
// in turn; a block is one wavefront.
__global__ __launch_bounds__(kWave, 5) void k_simulate_virtual(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                            EventsDev ev, SimOut out) {
    __shared__ VirtLds sm;
    int64_t next = blockIdx.x;                    // this block's next unit, counted from the first unit of the current class
    auto one_class = [&](auto width_tag, int cls) {
        constexpr int R = decltype(width_tag)::value, kGroups = kWave / R;
        int64_t pos_lo, pos_end;
        interleaved_range(ws, cls, pos_lo, pos_end);
        const int64_t units = (pos_end - pos_lo + kGroups - 1) / kGroups;
        for (; next < units; next += gridDim.x)
            virtual_unit<R>(co, cl, ca, ws, ev, out, pos_lo + next * kGroups, pos_end, sm);
        next -= units;
    };
    static_assert(kClasses == 7, "one call per class below");
    one_class(std::integral_constant<int, 64>{}, 0);
    one_class(std::integral_constant<int, 32>{}, 1);
    one_class(std::integral_constant<int, 16>{}, 2);
    one_class(std::integral_constant<int, 8>{}, 3);
    one_class(std::integral_constant<int, 4>{}, 4);
    one_class(std::integral_constant<int, 2>{}, 5);
    one_class(std::integral_constant<int, 2>{}, 6);
}

// Timeline dump of the selected candidates that use the interleaved schedule; one wavefront per
// selection.  The block of candidate sel[q] holds 2 * pp * chunks * m entries laid out
// [kind][virtual stage][micro-batch]; the all-reduce windows are per device.  Runs after
// k_timeline, which has set every all-reduce window to -1 and skipped these candidates.
__global__ __launch_bounds__(kWave) void k_timeline_virtual(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                            const int32_t* status, int64_t C, int64_t n,
                                                            const int64_t* sel, const int64_t* task_off,
                                                            int64_t* start_ns, int64_t* end_ns, int64_t* ar_start,
                                                            int64_t* ar_end) {
    __shared__ VirtLds sm;
    for (int64_t q = blockIdx.x; q < n; q += gridDim.x) {
        const int64_t c = sel[q];
        if (c < 0 || c >= C || status[c] != 0 || ca.schedule[c] != 3 || !ca.chunks) continue;
        const int tp = ca.tp[c];
        int v = -1;
        for (int i = 0; i < co.V; i++)
            if (co.variant_tp[i] == tp) { v = i; break; }
        if (v < 0) continue;                                              // cannot be: the status is OK
        const VirtCand vc{ca.pp[c], v, ca.m[c], ca.dp[c], tp, ca.chunks[c], 0, ca.part_off[c], c};
        const int64_t off = task_off[q];
        const VirtDump dump{start_ns + off, end_ns + off, ar_start + q * kMaxPP, ar_end + q * kMaxPP};
        virtual_groups<true, kWave>(co, cl, ca, ws, EventsDev{}, SimOut{}, vc, dump, sm);
        __syncthreads();
    }
}

}  // namespace distsim
