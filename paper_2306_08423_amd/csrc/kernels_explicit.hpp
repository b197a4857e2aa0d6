// Explicit schedules: the device lists of Algorithm 1's schedule S given by the caller (Sec. 4.3),
// the door through which a new pipeline algorithm enters (Sec. 7).  One wavefront per candidate,
// lane = device (for the set-up also lane = virtual stage).  The end of every task that has run
// is kept in LDS by (kind, stage, micro-batch); per round every lane looks at the next task of
// its list and runs it if its input is there: start = max(device free, end of the producing task
// + p2p event), the rule of Algorithm 1.  A round in which no lane can run a task ends the loop:
// the schedule cannot be run to its end and the candidate is invalid.  Same arithmetic as the
// level sweeps: fp64 values that are integers below 2^53.  The slow path: generality, not speed
// (the schedules that get a program, nearly all, run through kernels_schedule.hpp instead).
#pragma once
#include "kernels_virtual.hpp"

namespace distsim {

// LDS of one candidate of at most SLOTS (virtual stage, micro-batch) pairs.
template <int SLOTS>
struct ExplicitLds {
    // first index: kind of the task, 0 = forward, 1 = backward
    double end[2][SLOTS];                       // end of the task, kNotListed / kListed before it has run
    double dur[2][kMaxPP];                      // by virtual stage: task durations
    double lat[2][kMaxPP];                      // by virtual stage: latency of the incoming edge
    int64_t send[2][kMaxPP];                    // by virtual stage: outgoing p2p events
    int64_t comp[2][kMaxPP];                    // by virtual stage: computation inside a task
    int64_t comm[2][kMaxPP];                    // by virtual stage: communication inside a task and its outgoing p2p event
    int64_t grad[kMaxPP];                       // by virtual stage: gradient bytes of its part
    int32_t place[kMaxPP], prev[kMaxPP], next[kMaxPP], succ[kMaxPP];
    // p2p_blocking = 2: a link is an ordered pair (sending device, receiving device) and carries one
    // transfer at a time.  link[kind][k]: the queue that the send after a task of (kind, stage k)
    // uses = the lowest-numbered edge between the same two devices (kind * kMaxPP + stage);
    // link_free[queue]: arrival of the latest transfer on it.  Only the sending device's lane
    // touches a queue.
    int32_t link[2][kMaxPP];
    double link_free[2 * kMaxPP];
    double send_d[2][kMaxPP];                   // outgoing p2p events as doubles
};
constexpr double kNotListed = -1.0, kListed = -2.0;

// What one candidate needs from its descriptor (or, for the dump, from the candidate arrays).
struct ExplicitCand {
    int pp, v, m, dp, tp;
    int64_t id, poff, c;
};

// One candidate on one wavefront.  DUMP = false: writes status / batch time / busy sums.
// DUMP = true: the candidate is known to be OK; writes the start and end of every listed task
// ([kind][virtual stage][micro-batch], -1 for tasks that are not listed) and the all-reduce
// windows, and none of the simulation's outputs.
template <bool DUMP, typename Lds>
__device__ __forceinline__ void explicit_candidate(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                                   const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                                   const ExplicitCand& xc, const VirtDump& dump, Lds& sm) {
    const int lane = threadIdx.x;
    const int L = co.L;
    __syncthreads();                                                  // the previous candidate's LDS is free
    const int pp = xc.pp, v = xc.v, m = xc.m, dp = xc.dp, tp = xc.tp;
    const int64_t id = xc.id, c = xc.c;
    auto invalid = [&]() {
        if (!DUMP && lane == 0) { ev.status[c] = 1; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
    };
    // k_decode has checked the head of the block (pp, m, S, nparts, replicas, S * m)
    const int64_t woff = ca.schedule_off[id], nwords = ca.schedule_off[id + 1] - woff;
    const int32_t* w = ca.schedule_words + woff;
    const int S = w[1], nparts = w[3], replicas = w[4];
    const int32_t* dev_off = w + 5;
    const int64_t ntask = dev_off[pp];
    bool bad = dev_off[0] != 0 || ntask < 0 || ntask > 2ll * S * m || nwords != 5 + pp + 1 + 3ll * S + ntask;
    const int t0 = lane < pp ? dev_off[lane] : 0, t1 = lane < pp ? dev_off[lane + 1] : 0;      // this device's list
    bad = bad || __builtin_amdgcn_ballot_w64(t1 < t0) != 0;
    if (bad) { invalid(); return; }
    const int32_t* st = dev_off + pp + 1;
    const int32_t* tasks = st + 3 * S;

    // the stages (lane = virtual stage)
    const bool isk = lane < S;
    int place = 0, part = 0, prev = -1;
    if (isk) { place = st[3 * lane]; part = st[3 * lane + 1]; prev = st[3 * lane + 2]; }
    bool kbad = isk && (place < 0 || place >= pp || part < 0 || part >= nparts || prev < -1 || prev >= S || prev == lane);
    sm.succ[lane] = 0;
    sm.next[lane] = -1;
    __syncthreads();
    if (isk && !kbad && prev >= 0) atomicAdd(&sm.succ[prev], 1);
    __syncthreads();
    kbad = kbad || (isk && sm.succ[lane] > 1);                        // at most one stage after any stage
    // the partition (lane = part): 0 = b0 < b1 < ... = L
    int plo = 0, phi = 0;
    if (lane < nparts) {
        if (xc.poff >= 0) { plo = ca.part_pool[xc.poff + lane]; phi = ca.part_pool[xc.poff + lane + 1]; }
        else { plo = uniform_bound(lane, L, nparts); phi = uniform_bound((lane + 1), L, nparts); }
        if (phi <= plo || phi > L || (lane == 0 && plo != 0) || (lane == nparts - 1 && phi != L)) kbad = true;
    }
    if (__builtin_amdgcn_ballot_w64(kbad) != 0) { invalid(); return; }
    if (isk && prev >= 0) sm.next[prev] = lane;
    if (isk) { sm.place[lane] = place; sm.prev[lane] = prev; }
    __syncthreads();

    // every task at most once, on the device of its stage; succ[] has done its work and now takes,
    // by stage, the place in the list of the stage's last backward task (-1 = none): that is the
    // task in which the stage's gradients are complete (bucketed all-reduce)
    const int slots = S * m;
    for (int i = lane; i < slots; i += kWave) { sm.end[0][i] = kNotListed; sm.end[1][i] = kNotListed; }
    sm.succ[lane] = -1;
    __syncthreads();
    bool lbad = false;
    for (int i = t0; i < t1; i++) {
        const uint32_t x = (uint32_t)tasks[i];
        const int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;
        if (k >= S || j >= m || sm.place[k] != lane) { lbad = true; break; }
        double* e = sm.end[kd] + k * m + j;                             // only this lane holds stage k
        if (*e != kNotListed) { lbad = true; break; }
        *e = kListed;
        if (kd) sm.succ[k] = i;
    }
    if (__builtin_amdgcn_ballot_w64(lbad) != 0) { invalid(); return; }
    __syncthreads();


    // composed events of every stage's part, p2p events of the edges
    const int64_t tpdp = (int64_t)tp * dp;
    auto node_of = [&](int dev) -> int64_t {
        return tpdp >= cl.gpus_per_node ? dev : (int64_t)node_of_position(cl, dev, (int)tpdp);
    };
    const int64_t* row = ws.comb + (size_t)((v * kMaxPP + pp - 1) * (L + 1)) * kCombWords;
    const size_t vr = (size_t)v * (L + 1);
    int64_t FT = 0, BT = 0, PB = 0, share = 0;
    sm.send[0][lane] = 0;
    __syncthreads();
    if (isk) {
        int lo, hi;
        if (xc.poff >= 0) { lo = ca.part_pool[xc.poff + part]; hi = ca.part_pool[xc.poff + part + 1]; }
        else { lo = uniform_bound(part, L, nparts); hi = uniform_bound((part + 1), L, nparts); }
        const int64_t* eh = row + hi * kCombWords;
        const int64_t* el = row + lo * kCombWords;
        FT = eh[0] - el[0]; BT = eh[1] - el[1];
        const int64_t fcp = ws.pfc[vr + hi] - ws.pfc[vr + lo], bcp = ws.pbc[vr + hi] - ws.pbc[vr + lo];
        sm.comp[0][lane] = fcp; sm.comp[1][lane] = bcp;
        sm.comm[0][lane] = FT - fcp; sm.comm[1][lane] = BT - bcp;
        sm.grad[lane] = eh[3] - el[3];
        if (prev >= 0) {
            // the activation that leaves the part of the stage before: entry of the layer after it
            const int pq = st[3 * prev + 1];
            int qhi;
            if (xc.poff >= 0) qhi = ca.part_pool[xc.poff + pq + 1];
            else qhi = uniform_bound((pq + 1), L, nparts);
            const int inter = node_of(sm.place[prev]) != node_of(place) ? 1 : 0;
            PB = row[qhi * kCombWords + 4 + inter];
            sm.send[0][prev] = PB;                                   // the same event, sent forwards by the stage before
        }
        sm.send[1][lane] = PB;
    }
    __syncthreads();
    if (isk) share = FT + BT + sm.send[0][lane] + PB;
    if (stage_out_of_range(isk ? share : 0, m, kWave)) {
        if (!DUMP && lane == 0) { ev.status[c] = 2; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        return;
    }
    if (isk) {
        const int64_t pf_task = cl.blocking == 1 ? sm.send[0][lane] : 0, pb_task = cl.blocking == 1 ? PB : 0;
        sm.dur[0][lane] = (double)(FT + pf_task);
        sm.dur[1][lane] = (double)(BT + pb_task);
        sm.comm[0][lane] += sm.send[0][lane];
        sm.comm[1][lane] += PB;
    }
    __syncthreads();
    if (isk) {
        const int nx = sm.next[lane];
        // latency of the incoming edge; none when the send is part of the sender's task (1) or when
        // the consumer reads the transfer's arrival time instead of the task's end (2)
        sm.lat[0][lane] = prev >= 0 && cl.blocking == 0 ? (double)sm.send[0][prev] : 0.0;
        sm.lat[1][lane] = nx >= 0 && cl.blocking == 0 ? (double)sm.send[1][nx] : 0.0;
        sm.send_d[0][lane] = (double)sm.send[0][lane];
        sm.send_d[1][lane] = (double)sm.send[1][lane];
        if (cl.blocking == 2) {
            // the queue of each of the stage's two outgoing edges: forward to next, backward to prev
            const int dst_f = nx >= 0 ? sm.place[nx] : -1, dst_b = prev >= 0 ? sm.place[prev] : -1;
            int qf = lane, qb = kMaxPP + lane;
            for (int k2 = 0; k2 < S; k2++) {
                if (sm.place[k2] != place) continue;
                const int n2 = sm.next[k2], p2 = sm.prev[k2];
                const int d2f = n2 >= 0 ? sm.place[n2] : -1, d2b = p2 >= 0 ? sm.place[p2] : -1;
                if (d2f >= 0 && d2f == dst_f && k2 < qf) qf = k2;
                if (d2f >= 0 && d2f == dst_b && k2 < qb) qb = k2;
                if (d2b >= 0 && d2b == dst_f && kMaxPP + k2 < qf) qf = kMaxPP + k2;
                if (d2b >= 0 && d2b == dst_b && kMaxPP + k2 < qb) qb = kMaxPP + k2;
            }
            sm.link[0][lane] = qf;
            sm.link[1][lane] = qb;
        }
    }
    sm.link_free[lane] = 0.0;
    sm.link_free[kMaxPP + lane] = 0.0;
    __syncthreads();
    if (DUMP) {                                                      // tasks that are not listed read -1
        for (int q = lane; q < 2 * slots; q += kWave) { dump.start[q] = -1; dump.end[q] = -1; }
    }

    // the rounds.  The word of the task after the next one is requested a task ahead, and all of a
    // round's LDS reads are issued together (at valid addresses whatever the task), so that a round
    // waits for one trip to LDS and not for the list in memory.
    int i = t0;
    uint32_t x = i < t1 ? (uint32_t)tasks[i] : 0u, xn = i + 1 < t1 ? (uint32_t)tasks[i + 1] : 0u;
    double own = 0.0;
    int64_t comp = 0, comm = 0, nsend = 0;
    bool stuck = false;
    for (int64_t round = 0; round <= ntask; round++) {
        const bool todo = i < t1;
        if (__builtin_amdgcn_ballot_w64(todo) == 0) break;
        bool ran = false;
        if (todo) {
            const int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;
            // the task that feeds this one: the same micro-batch on the stage before (forward) or
            // after (backward); at the end of its pipeline a backward follows its own forward,
            // which this device ran
            const int pv = sm.prev[k], nx = sm.next[k];
            const int link = kd ? nx : pv;
            const bool turn = kd && link < 0;
            const bool has_prod = link >= 0 || turn;
            const double e = sm.end[turn ? 0 : kd][(link >= 0 ? link : k) * m + j];
            const double lat = sm.lat[kd][k], dur = sm.dur[kd][k];
            const int64_t cp = sm.comp[kd][k], cm = sm.comm[kd][k];
            const bool sends = (kd ? pv : nx) >= 0;                  // the task is followed by a transfer
            const int queue = sm.link[kd][k];
            const double free_at = sm.link_free[cl.blocking == 2 && sends ? queue : 0], send = sm.send_d[kd][k];
            ran = !has_prod || e >= 0.0;
            if (ran) {                                               // a round's reads of end[] come before its writes
                const double arrive = has_prod ? e + lat : 0.0;
                const double start = arrive > own ? arrive : own;
                own = start + dur;
                double seen = own;                                   // what the consuming task reads
                if (cl.blocking == 2 && sends) {                     // the transfer queues on its link
                    seen = (own > free_at ? own : free_at) + send;
                    sm.link_free[queue] = seen;
                }
                sm.end[kd][k * m + j] = seen;
                // bucketed all-reduce: the start of the stage's last backward takes the place of its
                // duration, which no later task needs
                if (kd && cl.bucket > 0 && i == sm.succ[k]) sm.dur[1][k] = start;
                if (DUMP) {
                    const int64_t q = ((int64_t)kd * S + k) * m + j;
                    dump.start[q] = double_to_i64(start);
                    dump.end[q] = double_to_i64(own);
                }
                comp += cp;
                comm += cm;
                nsend += (kd ? pv : nx) >= 0 ? 1 : 0;
                i++;
                x = xn;
                xn = i + 1 < t1 ? (uint32_t)tasks[i + 1] : 0u;
            }
        }
        if (__builtin_amdgcn_ballot_w64(ran) == 0) { stuck = true; break; }
        __syncthreads();
    }
    if (stuck || __builtin_amdgcn_ballot_w64(i < t1) != 0) { invalid(); return; }

    // data-parallel modelling per device: one all-reduce after its list, over the bytes of all its
    // stages; or, with a bucket size, the device's buckets: a stage's gradients are complete in its
    // last backward task on the list, layer by layer from the last layer of its part down, each at the
    // start of that task + the backward events down to the layer; the device walks its list once more
    // to take those tasks in order; full buckets are issued at once and queue, the rest goes after the
    // device's last gradient; a stage without a backward task adds nothing.
    const bool dev = lane < pp;
    const int64_t ranks = (int64_t)dp * replicas;
    const int64_t endL = double_to_i64(own);
    int64_t AR = 0, ar_first = endL, ar_last = endL, nar_dev = 0;                   // AR: busy time of the all-reduce events
    bool has_ar = false;
    if (cl.bucket <= 0) {
        int64_t G = 0;
        if (dev)
            for (int k = 0; k < S; k++)
                if (sm.place[k] == lane) G += sm.grad[k];
        has_ar = dev && t1 > t0 && ranks > 1 && G > 0;
        if (has_ar) { AR = allreduce_ns(cl, ranks, G); ar_last = endL + AR; nar_dev = 1; }
    } else if (dev && ranks > 1) {
        const int64_t ar_cap = allreduce_ns(cl, ranks, cl.bucket);
        int64_t t_free = 0, acc = 0, ready = 0;
        ar_first = -1;
        for (int q = t0; q < t1; q++) {
            const uint32_t y = (uint32_t)tasks[q];
            const int k = (y >> 16) & 0x7fff;
            if (!(y >> 31) || sm.succ[k] != q) continue;
            const int part_k = st[3 * k + 1];
            int lo, hi;
            if (xc.poff >= 0) { lo = ca.part_pool[xc.poff + part_k]; hi = ca.part_pool[xc.poff + part_k + 1]; }
            else { lo = uniform_bound(part_k, L, nparts); hi = uniform_bound((part_k + 1), L, nparts); }
            const int64_t startB = double_to_i64(sm.dur[1][k]), tot_hi = row[hi * kCombWords + 1];
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
            const int64_t b0 = t_free > ready ? t_free : ready, dd = allreduce_ns(cl, ranks, acc);
            if (ar_first < 0) ar_first = b0;
            t_free = b0 + dd;
            AR += dd; nar_dev++;
        }
        has_ar = nar_dev > 0;
        if (has_ar) ar_last = t_free;
    }
    if (DUMP) {
        if (has_ar) { dump.ar_start[lane] = ar_first; dump.ar_end[lane] = ar_last; }
        return;
    }
    const int64_t batch = group_max(dev ? (ar_last > endL ? ar_last : endL) : 0, kWave);
    const int64_t nar = group_sum(dev ? nar_dev : 0, kWave);
    const int64_t sends = group_sum(dev ? nsend : 0, kWave);
    const int64_t base = ev.stage_pos[c];
    if (dev && base >= 0) {
        out.comp_busy[base + lane] = comp;
        out.comm_busy[base + lane] = comm + AR;
        if (out.util) out.util[base + lane] = batch > 0 ? (double)comp / (double)batch : 0.0;
    }
    if (lane == 0) {
        out.batch_ns[c] = batch;
        ev.num_events[c] = ntask + sends + nar;
    }
}

// The candidates whose schedule k_compile_schedules left without a program (none as a rule: every
// block ends at once then); one wavefront per candidate, LDS for the largest schedule.  Walks the
// whole visiting order.
__global__ __launch_bounds__(kWave) void k_simulate_explicit(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                             EventsDev ev, SimOut out) {
    __shared__ ExplicitLds<kMaxSlots> sm;
    if (ws.hdr[H_SCHED_TABLE] == 0) return;
    // descriptors beyond the valid candidates were never written: the class table bounds them
    const int64_t pos_end = ws.hdr[H_CLASS_START + kClasses];
    for (int64_t pos = blockIdx.x; pos < pos_end; pos += gridDim.x) {
        const Desc ds = ws.desc[pos];
        if (!is_explicit(ds) || (ds.meta & 0xff) == 0) continue;          // uniform: one descriptor per wavefront
        const ExplicitCand xc{ds.meta & 0xff, ds.meta >> 16, ds.m, ds.dp, (int)(uint32_t)ds.spare, ds.spare >> 32, ds.poff,
                              ds.cand};
        if (xc.id < kSchedCap && ws.sched_hdr[xc.id].state != 0) continue;      // 0: no program
        // k_decode has checked the head of the block: 1 <= S <= 64, S * m <= kMaxSlots
        explicit_candidate<false>(co, cl, ca, ws, ev, out, xc, VirtDump{}, sm);
    }
}

// Timeline dump of the selected candidates that have an explicit schedule; one wavefront per
// selection.  The block of candidate sel[q] holds 2 * S * m entries laid out [kind][virtual stage]
// [micro-batch]; the all-reduce windows are per device.  Runs after k_timeline, which has set
// every all-reduce window to -1 and skipped these candidates.
__global__ __launch_bounds__(kWave) void k_timeline_explicit(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                             const int32_t* status, int64_t C, int64_t n,
                                                             const int64_t* sel, const int64_t* task_off,
                                                             int64_t* start_ns, int64_t* end_ns, int64_t* ar_start,
                                                             int64_t* ar_end) {
    __shared__ ExplicitLds<kMaxSlots> sm;
    for (int64_t q = blockIdx.x; q < n; q += gridDim.x) {
        const int64_t c = sel[q];
        if (c < 0 || c >= C || status[c] != 0 || ca.schedule[c] != 4 || !ca.chunks) continue;
        const int tp = ca.tp[c];
        int v = -1;
        for (int i = 0; i < co.V; i++)
            if (co.variant_tp[i] == tp) { v = i; break; }
        if (v < 0) continue;                                              // cannot be: the status is OK
        const ExplicitCand xc{ca.pp[c], v, ca.m[c], ca.dp[c], tp, ca.chunks[c], ca.part_off[c], c};
        const int64_t off = task_off[q];
        const VirtDump dump{start_ns + off, end_ns + off, ar_start + q * kMaxPP, ar_end + q * kMaxPP};
        explicit_candidate<true>(co, cl, ca, ws, EventsDev{}, SimOut{}, xc, dump, sm);
    }
}

}  // namespace distsim
