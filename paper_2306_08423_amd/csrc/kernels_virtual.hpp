// Interleaved one-forward-one-backward schedule: every device holds several model chunks, so a
// device's tasks belong to several virtual stages and the producer of a task is no longer "the
// neighbour's latest task".  A wavefront is cut into groups of R lanes, one candidate per group,
// lane = device.  Each lane walks its own task list (closed forms of the slot numbers, see
// distsim.h) and keeps the end times of its latest forward and backward slots in LDS rings; in
// every round a lane runs its next task if the producing slot on the neighbouring device (the
// device before for forwards, after for backwards, with the edge from the last device back to
// the first one chunk apart) has been run, reading its end time from that device's ring.  Rounds
// repeat until every list of the wavefront is done; a round in which no lane can run ends the
// loop (it cannot happen for a valid schedule) and the candidates still unfinished are reported
// invalid.  Same arithmetic as the level sweep: fp64 values that are integers below 2^53.
#pragma once
#include "kernels_simulate.hpp"

namespace distsim {

// LDS of one wavefront: 64 / R candidates of at most R devices each, R ring slots per device and
// direction.  A producer never leads its consumer by more than the ring holds when R >= max(8, pp)
// (checked by running the rounds, which do not depend on the durations, for every pp, every chunk
// count with pp * chunks <= 64 and micro-batch counts up to 8 pp); a task that would overwrite a
// slot not yet read waits, so a ring that were too small could stall a candidate but never give
// a wrong time.
template <int R>
struct VirtLds {
    static_assert(R >= 8 && R <= kWave && (R & (R - 1)) == 0, "ring sizes are powers of two from 8 to 64");
    static constexpr int kRing = R, kGroups = kWave / R;
    // first index: direction, 0 = forward, 1 = backward
    union {
        double ring[2][kWave][R];               // by lane and slot modulo R: end of the task
        // by group and virtual stage: outgoing p2p events; needed only while the latencies are
        // set up, before the first round writes the rings (64 R >= (64 / R) 64 entries for R >= 8)
        int64_t send[2][kGroups][kMaxPP];
    };
    double dur[2][kGroups][kMaxPP];             // by group and virtual stage: task durations
    double lat[2][kGroups][kMaxPP];             // by group and virtual stage: latency of the incoming edge
    int32_t done[2][kWave];                     // by lane: slots run, as of the previous round
};

// What one candidate needs from its descriptor (or, for the dump, from the candidate arrays); the
// lanes of a group hold the same values.  pp == 0: the group has no candidate.
struct VirtCand {
    int pp, v, m, dp, tp, vch;
    int64_t poff, c;
};

// Where the dump of one candidate goes (the simulation proper passes none).
struct VirtDump {
    int64_t* start;      // [2][pp * vch][m]
    int64_t* end;
    int64_t* ar_start;   // [kMaxPP] by device
    int64_t* ar_end;
};

// The candidates of one wavefront, one per group of Lds::kRing lanes.  DUMP = false: writes status
// / batch time / busy sums.  DUMP = true: the candidates are known to be OK; writes every task's
// start and end and the all-reduce windows, and none of the simulation's outputs.
template <bool DUMP, typename Lds>
__device__ __forceinline__ void virtual_groups(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                               const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                               const VirtCand& vc, const VirtDump& dump, Lds& sm) {
    constexpr int R = Lds::kRing;
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
            sm.dur[0][g][k] = (double)(FT + pf_task);
            sm.dur[1][g][k] = (double)(BT + pb_task);
            sm.send[0][g][k] = PF - pf_task;
            sm.send[1][g][k] = PB - pb_task;
        }
    }
    const bool gbad = group_any(bad != 0, R);
    const bool range = stage_out_of_range(act && !gbad ? share : 0, m, R);
    if (gbad || range) {
        if (!DUMP && act && d == 0) { ev.status[c] = gbad ? 1 : 2; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        act = false;
    }
    __syncthreads();
    // latency of the edge into virtual stage k: the send of k - 1 (forward), of k + 1 (backward)
    if (act) {
        for (int cch = 0; cch < vch; cch++) {
            const int k = cch * pp + d;
            sm.lat[0][g][k] = k > 0 ? (double)sm.send[0][g][k - 1] : 0.0;
            sm.lat[1][g][k] = k + 1 < S ? (double)sm.send[1][g][k + 1] : 0.0;
        }
    }
    __syncthreads();

    // the rounds
    // slot numbers fit 32 bits: m <= 2^16 and pp * vch <= 64
    const int n = act ? m * vch : 0;                          // slots per direction
    int W = 2 * (pp - d - 1) + (vch - 1) * pp;                // warm-up forwards
    if (W > n) W = n;
    int iF = 0, iB = 0;
    // slot i of a direction = group (i / (pp vch)), position of the chunk (i mod (pp vch)) / pp,
    // place in the chunk i mod pp; kept as counters: r, c and the group's first micro-batch
    int rF = 0, cF = 0, rB = 0, cB = 0;
    int jF0 = 0, jB0 = 0;
    double own = 0.0;
    // p2p_blocking = 2: a link is an ordered pair (sending device, receiving device) and carries one
    // transfer at a time.  A device sends forwards to the device after it and backwards to the one
    // before it (both modulo pp): two queues, which are one and the same for pp <= 2.
    double link_f = 0.0, link_b = 0.0;
    const bool one_queue = pp <= 2;
    const int max_rounds = wave_max_i32(act ? 4 * n + 8 * pp + 64 : 0);
    // Per direction: the producer of a slot is the same slot on the device before (in the
    // direction), or, on the direction's first device, the slot pp earlier on its last device; the
    // consumers of the ring slot that a task overwrites are the device after and, on the
    // direction's last device, the first device (pp slots later).  All of a round's LDS reads are
    // issued together, at clamped addresses, and the conditions select among what came back.
    const int dL = g0 + (d > 0 ? d - 1 : 0), dR = g0 + (d + 1 < pp ? d + 1 : d);      // neighbouring lanes
    const int dFirst = g0, dLast = g0 + (pp > 0 ? pp - 1 : 0);
    for (int round = 0; round < max_rounds; round++) {
        if (act) { sm.done[0][lane] = iF; sm.done[1][lane] = iB; }
        __syncthreads();
        const bool todo = act && iB < n;
        if (__builtin_amdgcn_ballot_w64(todo) == 0) break;
        bool ran = false;
        if (todo) {
            const bool fwd = iF < W || (iF < n && iF - W == iB);
            const int dir = fwd ? 0 : 1;
            const int i = fwd ? iF : iB;
            // chunk and micro-batch of the slot, from the counters kept with iF / iB
            const int cch = fwd ? cF : vch - 1 - cB;
            const int k = cch * pp + d;
            const bool has_prod = fwd ? k > 0 : k + 1 < S;
            const bool first = fwd ? d == 0 : d + 1 == pp;            // first device of the direction
            const bool last = fwd ? d + 1 == pp : d == 0;             // last device of the direction
            const int src = first ? (fwd ? dLast : dFirst) : (fwd ? dL : dR);
            const int si = first ? i - pp : i;
            const int done_src = sm.done[dir][src];
            const double prod_end = sm.ring[dir][src][si & (R - 1)];
            const double lat = sm.lat[dir][g][k], dur = sm.dur[dir][g][k];
            const bool sends = fwd ? k + 1 < S : k > 0;                // the task is followed by a transfer ...
            const double send = sm.lat[dir][g][sends ? (fwd ? k + 1 : k - 1) : k];      // ... which is the consumer's edge
            const int done_next = sm.done[dir][fwd ? dR : dL];
            const int done_wrap = sm.done[dir][fwd ? dFirst : dLast];
            bool ok = !has_prod || done_src > si;
            // the slot this task overwrites in the ring must have been read by its consumers
            if (i >= R) {
                if (!last && !(done_next > i - R)) ok = false;
                if (last && vch > 1 && !(done_wrap > i - R + pp)) ok = false;
            }
            if (ok) {
                // with queues on the links the producer has stored the transfer's arrival time
                const double arrive = has_prod ? prod_end + (cl.blocking == 2 ? 0.0 : lat) : 0.0;
                const double t0 = arrive > own ? arrive : own;
                own = t0 + dur;
                double seen = own;                                     // what the consuming task reads
                if (cl.blocking == 2 && sends) {
                    const bool q_f = fwd || one_queue;
                    const double free_at = q_f ? link_f : link_b;
                    seen = (own > free_at ? own : free_at) + send;
                    if (q_f) link_f = seen; else link_b = seen;
                }
                sm.ring[dir][lane][i & (R - 1)] = seen;
                const int j = fwd ? jF0 + rF : jB0 + rB;                        // micro-batch of the slot
                // bucketed all-reduce: the chunk's gradients are complete in this task; its duration is
                // not needed again (the chunk has no later backward), so the start time takes its place
                if (!fwd && j == m - 1 && cl.bucket > 0) sm.dur[1][g][k] = t0;
                if (fwd) {
                    iF++;
                    if (++rF == pp) { rF = 0; if (++cF == vch) { cF = 0; jF0 += pp; } }
                } else {
                    iB++;
                    if (++rB == pp) { rB = 0; if (++cB == vch) { cB = 0; jB0 += pp; } }
                }
                if (DUMP) {
                    const int64_t e = ((int64_t)dir * S + k) * m + j;
                    dump.start[e] = double_to_i64(t0);
                    dump.end[e] = double_to_i64(own);
                }
                ran = true;
            }
        }
        if (__builtin_amdgcn_ballot_w64(ran) == 0) break;               // nothing can run any more
        __syncthreads();
    }
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
            const int64_t startB = double_to_i64(sm.dur[1][g][k]), tot_hi = row[hi * kCombWords + 1];
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

// One launch per ring size R: the candidates of the classes [cls_lo, cls_hi) of the visiting order
// (class k holds the candidates of 64 >> k lanes, i.e. pp <= 64 >> k <= R), 64 / R consecutive
// ones per wavefront, so that candidates of few devices share a wavefront and take little LDS.
// Neighbours in visiting order have about the same number of micro-batches, hence lists of about
// the same length when their chunk counts agree.
template <int R>
__global__ __launch_bounds__(kWave) void k_simulate_virtual(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                            EventsDev ev, SimOut out, int cls_lo, int cls_hi) {
    constexpr int kGroups = kWave / R;
    __shared__ VirtLds<R> sm;
    const int g = threadIdx.x / R;
    // descriptors beyond the valid candidates were never written: the class table bounds them
    const int64_t pos_end = ws.hdr[H_CLASS_START + cls_hi];
    for (int64_t pos0 = ws.hdr[H_CLASS_START + cls_lo] + (int64_t)blockIdx.x * kGroups; pos0 < pos_end;
         pos0 += (int64_t)gridDim.x * kGroups) {
        Desc ds{};
        if (pos0 + g < pos_end) ds = ws.desc[pos0 + g];
        if (!is_interleaved(ds)) ds.meta = 0;
        if (__builtin_amdgcn_ballot_w64((ds.meta & 0xff) != 0) == 0) continue;
        const VirtCand vc{ds.meta & 0xff, ds.meta >> 16, ds.m, ds.dp, (int)(uint32_t)ds.spare, (int)(ds.spare >> 32),
                          ds.poff, ds.cand};
        virtual_groups<false>(co, cl, ca, ws, ev, out, vc, VirtDump{}, sm);
        __syncthreads();
    }
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
    __shared__ VirtLds<kMaxPP> sm;
    for (int64_t q = blockIdx.x; q < n; q += gridDim.x) {
        const int64_t c = sel[q];
        if (c < 0 || c >= C || status[c] != 0 || ca.schedule[c] != 3 || !ca.chunks) continue;
        const int tp = ca.tp[c];
        int v = -1;
        for (int i = 0; i < co.V; i++)
            if (co.variant_tp[i] == tp) { v = i; break; }
        if (v < 0) continue;                                              // cannot be: the status is OK
        const VirtCand vc{ca.pp[c], v, ca.m[c], ca.dp[c], tp, ca.chunks[c], ca.part_off[c], c};
        const int64_t off = task_off[q];
        const VirtDump dump{start_ns + off, end_ns + off, ar_start + q * kMaxPP, ar_end + q * kMaxPP};
        virtual_groups<true>(co, cl, ca, ws, EventsDev{}, SimOut{}, vc, dump, sm);
        __syncthreads();
    }
}

}  // namespace distsim
