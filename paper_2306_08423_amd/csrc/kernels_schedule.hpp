// Explicit schedules, the fast path.  Which task of a schedule S (Sec. 4.3, Algorithm 1) can run
// when depends on the device lists and the stage graph alone, not on the durations: running the
// lists round by round (every device runs its next task if the producing task ran in an earlier
// round) gives every task a round number that holds for every candidate that uses the schedule.
// k_compile_schedules does that once per schedule, at event generation, and writes a program:
// per task its round, whether and where it reads its producer's end and where it leaves its own
// (a slot of a small ring per stage and kind, as deep as the schedule needs), plus per stage what
// the candidates need of the stage graph.  k_simulate_scheduled then runs a candidate without any
// test of readiness and without the table of all task ends: lane = device, 64 / R candidates per
// wavefront, a few KB of LDS for all of them.  Schedules that do not fit the program's limits keep
// the kernel with the full table (k_simulate_explicit); invalid ones are marked as such here.
#pragma once
#include "kernels_explicit.hpp"

namespace distsim {

constexpr int kSchedMaxDepth = 16;             // deepest ring a program may ask for
// kSchedInvalid: a malformed block or list (no strategy, whatever the candidate); kSchedStuck: well-formed lists
// that cannot be run to their ends (no strategy either, but a candidate's own checks come first)
enum : int32_t { kSchedTable = 0, kSchedCompiled = 1, kSchedInvalid = 2, kSchedStuck = 3 };

// A task of a compiled schedule (one 64-bit word, at the place of the task's word in the block).
//   bits  0-15 round            16-21 stage        22 kind (1 = backward)
//         23 reads a producer   24 has a consumer  25 last backward of its stage on the list
//         32-43 slot read       44-55 slot written (entries of the candidate's ring pool)
__device__ __forceinline__ int op_round(uint64_t op) { return (int)(op & 0xffff); }
__device__ __forceinline__ int op_stage(uint64_t op) { return (int)(op >> 16 & 63); }
__device__ __forceinline__ int op_kind(uint64_t op) { return (int)(op >> 22 & 1); }
constexpr uint64_t kOpReads = 1ull << 23, kOpFeeds = 1ull << 24, kOpLastBwd = 1ull << 25;
__device__ __forceinline__ int op_read_slot(uint64_t op) { return (int)(op >> 32 & 0xfff); }
__device__ __forceinline__ int op_write_slot(uint64_t op) { return (int)(op >> 44 & 0xfff); }

// What a candidate needs of stage k, at the places of the stage's three words in the block:
//   word 0: prev | next << 8 (0xff = none) | device << 16 | queue of the forward send << 24 |
//           queue of the backward send << 32 | layer part << 40
//           (queues: p2p_blocking = 2, index into the candidate's 2 S link queues)
//   word 1: forward tasks on the list | backward tasks on the list << 16
__device__ __forceinline__ int info_prev(uint64_t w) { const int x = (int)(w & 0xff); return x == 0xff ? -1 : x; }
__device__ __forceinline__ int info_next(uint64_t w) { const int x = (int)(w >> 8 & 0xff); return x == 0xff ? -1 : x; }
__device__ __forceinline__ int info_place(uint64_t w) { return (int)(w >> 16 & 0xff); }
__device__ __forceinline__ int info_queue(uint64_t w, int kd) { return (int)(w >> (kd ? 32 : 24) & 0xff); }
__device__ __forceinline__ int info_part(uint64_t w) { return (int)(w >> 40 & 0xffff); }

struct CompileLds {
    // first index: kind of the task, 0 = forward, 1 = backward; second: stage * m + micro-batch
    int16_t rnd[2][kMaxSlots];                  // round in which the task ran, -1 before
    int16_t seq[2][kMaxSlots];                  // its place among the tasks of its stage and kind that have run
    int16_t byseq[2][kMaxSlots];                // by stage * m + place: the micro-batch
    uint32_t words[2 * kMaxSlots];              // the lists
    int32_t place[kMaxPP], prev[kMaxPP], next[kMaxPP], succ[kMaxPP], part[kMaxPP];
    int32_t count[2][kMaxPP];                   // tasks of the stage and kind that have run
    int32_t lastb[kMaxPP];                      // by stage: place in the list of its latest backward
    int32_t link[2][kMaxPP];
};

// One wavefront per schedule.  The checks are those of explicit_candidate, which this kernel
// takes over for the schedules it compiles; lane = device in the rounds, = stage before.
__global__ __launch_bounds__(kWave) void k_compile_schedules(CandDev ca, Workspace ws) {
    __shared__ CompileLds sm;
    const int lane = threadIdx.x;
    const int64_t ids = ca.n_schedules < kSchedCap ? ca.n_schedules : kSchedCap;
    if (blockIdx.x == 0 && lane == 0 && ca.n_schedules > kSchedCap)
        atomicAdd((unsigned long long*)&ws.hdr[H_SCHED_TABLE], (unsigned long long)(ca.n_schedules - kSchedCap));
    for (int64_t id = blockIdx.x; id < ids; id += gridDim.x) {
        __syncthreads();                                                  // the previous schedule's LDS is free
        int state = kSchedCompiled, n_rounds = 0, depth = 0, n_send = 0;
        auto done = [&]() {
            if (lane == 0) {
                ws.sched_hdr[id] = SchedHdr{state, n_rounds, depth, n_send};
                if (state == kSchedTable) atomicAdd((unsigned long long*)&ws.hdr[H_SCHED_TABLE], 1ull);
            }
        };
        const int64_t woff = ca.schedule_off[id], nwords = ca.schedule_off[id + 1] - woff;
        // a block that is not there, or has no room for a head: no candidate passes k_decode with it
        // (written so that offsets near 2^63 cannot wrap the sum)
        if (woff < 0 || nwords < 6 || woff > ca.schedule_words_len || nwords > ca.schedule_words_len - woff) {
            state = kSchedInvalid; done(); continue;
        }
        const int32_t* w = ca.schedule_words + woff;
        const int pp = w[0], S = w[1], m = w[2], nparts = w[3];
        // beyond the program's limits (k_decode reports such candidates as beyond the library anyway)
        if (woff + nwords > kSchedOpsCap || pp < 1 || pp > kMaxPP || S < 1 || S > kMaxPP || m < 1 || nparts < 1 ||
            (int64_t)S * m > kMaxSlots || nwords < 5 + pp + 1) {
            state = kSchedTable; done(); continue;
        }
        uint64_t* ops = (uint64_t*)ws.sched_ops + woff;
        const int32_t* dev_off = w + 5;
        const int64_t ntask = dev_off[pp];
        bool bad = dev_off[0] != 0 || ntask < 0 || ntask > 2ll * S * m || nwords != 5 + pp + 1 + 3ll * S + ntask;
        const int t0 = lane < pp ? dev_off[lane] : 0, t1 = lane < pp ? dev_off[lane + 1] : 0;      // this device's list
        bad = bad || __builtin_amdgcn_ballot_w64(t1 < t0 || t0 < 0 || t1 > ntask) != 0;
        if (bad) { state = kSchedInvalid; done(); continue; }
        const int sb = 5 + pp + 1, tb = sb + 3 * S;
        const int32_t* st = w + sb;
        const int32_t* tasks = w + tb;

        // the stages (lane = stage)
        const bool isk = lane < S;
        int place = 0, part = 0, prev = -1;
        if (isk) { place = st[3 * lane]; part = st[3 * lane + 1]; prev = st[3 * lane + 2]; }
        bool kbad = isk && (place < 0 || place >= pp || part < 0 || part >= nparts || prev < -1 || prev >= S || prev == lane);
        sm.succ[lane] = 0;
        sm.next[lane] = -1;
        sm.count[0][lane] = 0; sm.count[1][lane] = 0;
        sm.lastb[lane] = -1;
        __syncthreads();
        if (isk && !kbad && prev >= 0) atomicAdd(&sm.succ[prev], 1);
        __syncthreads();
        kbad = kbad || (isk && sm.succ[lane] > 1);                        // at most one stage after any stage
        if (__builtin_amdgcn_ballot_w64(kbad) != 0) { state = kSchedInvalid; done(); continue; }
        if (isk && prev >= 0) sm.next[prev] = lane;
        if (isk) { sm.place[lane] = place; sm.prev[lane] = prev; sm.part[lane] = part; }
        const int slots = S * m;
        for (int i = lane; i < slots; i += kWave) { sm.rnd[0][i] = -1; sm.rnd[1][i] = -1; }
        for (int i = lane; i < (int)ntask; i += kWave) sm.words[i] = (uint32_t)tasks[i];
        __syncthreads();
        // p2p_blocking = 2: the queue of each of a stage's two outgoing edges = the lowest-numbered
        // edge between the same two devices (forward edges of the stages first, then backward ones)
        if (isk) {
            const int nx = sm.next[lane];
            const int dst_f = nx >= 0 ? sm.place[nx] : -1, dst_b = prev >= 0 ? sm.place[prev] : -1;
            int qf = lane, qb = S + lane;
            for (int k2 = 0; k2 < S; k2++) {
                if (sm.place[k2] != place) continue;
                const int n2 = sm.next[k2], p2 = sm.prev[k2];
                const int d2f = n2 >= 0 ? sm.place[n2] : -1, d2b = p2 >= 0 ? sm.place[p2] : -1;
                if (d2f >= 0 && d2f == dst_f && k2 < qf) qf = k2;
                if (d2f >= 0 && d2f == dst_b && k2 < qb) qb = k2;
                if (d2b >= 0 && d2b == dst_f && S + k2 < qf) qf = S + k2;
                if (d2b >= 0 && d2b == dst_b && S + k2 < qb) qb = S + k2;
            }
            sm.link[0][lane] = qf;
            sm.link[1][lane] = qb;
        }
        __syncthreads();
        // every task at most once, on the device of its stage (-2: listed)
        bool lbad = false;
        for (int q = t0; q < t1; q++) {
            const uint32_t x = sm.words[q];
            const int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;
            if (k >= S || j >= m || sm.place[k] != lane) { lbad = true; break; }
            int16_t* e = sm.rnd[kd] + k * m + j;                        // only this lane holds stage k
            if (*e != -1) { lbad = true; break; }
            *e = -2;
        }
        if (__builtin_amdgcn_ballot_w64(lbad) != 0) { state = kSchedInvalid; done(); continue; }
        if (isk)
            ops[sb + 3 * lane] = (uint64_t)(prev & 0xff) | (uint64_t)(sm.next[lane] & 0xff) << 8 | (uint64_t)place << 16 |
                                 (uint64_t)sm.link[0][lane] << 24 | (uint64_t)sm.link[1][lane] << 32 | (uint64_t)part << 40;
        __syncthreads();

        // the rounds (lane = device): a task runs if its producer ran in an earlier round; all of a
        // round's reads come before its writes
        int i = t0, sends = 0;
        bool dead = false;
        for (int round = 0; round <= (int)ntask; round++) {
            const bool todo = i < t1 && !dead;
            if (__builtin_amdgcn_ballot_w64(todo) == 0) { n_rounds = round; break; }
            bool ran = false;
            if (todo) {
                const uint32_t x = sm.words[i];
                const int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;       // checked above
                const int pv = sm.prev[k], nx = sm.next[k];
                const int link = kd ? nx : pv;
                const bool turn = kd && link < 0;
                const int prod = sm.rnd[turn ? 0 : kd][(link >= 0 ? link : k) * m + j];
                const int own_seq = sm.count[kd][k];
                ran = !(link >= 0 || turn) || prod >= 0;
                if (ran) {
                    const bool feeds = (kd ? pv : nx) >= 0;
                    sm.rnd[kd][k * m + j] = (int16_t)round;
                    sm.seq[kd][k * m + j] = (int16_t)own_seq;
                    sm.byseq[kd][k * m + own_seq] = (int16_t)j;
                    sm.count[kd][k] = own_seq + 1;
                    if (kd) sm.lastb[k] = i;
                    sends += feeds ? 1 : 0;
                    i++;
                }
            }
            if (__builtin_amdgcn_ballot_w64(ran) == 0) { dead = true; break; }                        // stuck
            __syncthreads();
        }
        // a list that did not end: the schedule cannot be run
        if (__builtin_amdgcn_ballot_w64(i < t1 || dead) != 0) { state = kSchedStuck; done(); continue; }
        __syncthreads();
        n_send = (int)group_sum(sends, kWave);

        // the ring depth: the n-th end of a stage and kind goes where the (n - depth)-th went, which
        // must have been read by then (in the same round at the latest: reads come first)
        for (depth = 1; depth <= kSchedMaxDepth; depth <<= 1) {
            bool fits = true;
            for (int q = lane; q < 2 * slots; q += kWave) {
                const int kd = q >= slots ? 1 : 0, e = q - kd * slots, k = e / m, n = e - k * m;
                const int cons = kd ? sm.prev[k] : sm.next[k];
                if (cons < 0 || n < depth || n >= sm.count[kd][k]) continue;
                const int written = sm.rnd[kd][k * m + sm.byseq[kd][k * m + n]];
                const int read = sm.rnd[kd][cons * m + sm.byseq[kd][k * m + n - depth]];
                if (read < 0 || read > written) fits = false;
            }
            if (__builtin_amdgcn_ballot_w64(!fits) == 0) break;
        }
        if (depth > kSchedMaxDepth || 2 * S * depth > kSchedMaxPool) { state = kSchedTable; depth = 0; done(); continue; }

        // the stages' task counts and the tasks (all lanes take the tasks in turn)
        if (isk) ops[sb + 3 * lane + 1] = (uint64_t)sm.count[0][lane] | (uint64_t)sm.count[1][lane] << 16;
        for (int q = lane; q < (int)ntask; q += kWave) {
            const uint32_t x = sm.words[q];
            const int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;
            const int pv = sm.prev[k], nx = sm.next[k];
            const int link = kd ? nx : pv;
            const bool feeds = (kd ? pv : nx) >= 0;
            const int rd = link >= 0 ? (kd * S + link) * depth + (sm.seq[kd][link * m + j] & (depth - 1)) : 0;
            const int wr = (kd * S + k) * depth + (sm.seq[kd][k * m + j] & (depth - 1));
            ops[tb + q] = (uint64_t)(uint16_t)sm.rnd[kd][k * m + j] | (uint64_t)k << 16 | (uint64_t)kd << 22 |
                          (link >= 0 ? kOpReads : 0) | (feeds ? kOpFeeds : 0) | (kd && sm.lastb[k] == q ? kOpLastBwd : 0) |
                          (uint64_t)rd << 32 | (uint64_t)wr << 44;
        }
        done();
    }
}

// LDS of one wavefront of k_simulate_scheduled: 64 / R candidates, which share the tables below
// (each takes S stages and 2 S depth ring entries; those that do not fit wait for a further pass).
struct SchedStage {                             // task durations; the latency added to the producer's end,
    double dur_f, add_f, dur_b, add_b;          // or, with link queues, the transfer that follows the task
};
struct SchedLds {
    static constexpr int kStages = kWave, kRing = 8, kBatch = 4;
    double pool[kSchedWavePool];                // ring entries: ends of tasks, as their consumers see them
    alignas(32) SchedStage st[kStages];
    int64_t own_p2p[kStages];                   // by stage: p2p event of the edge from its prev (set-up only)
    int32_t queue[kStages];                     // by stage: queue of the forward send | of the backward send << 8
    double link_free[2 * kStages];              // p2p_blocking = 2: arrival of the latest transfer on a queue
    double lastb_start[kStages];                // bucketed all-reduce: start of the stage's last backward
    unsigned long long dev_sum[3][kWave];       // by lane = device: computation, communication, gradient bytes of its stages
    uint64_t ops[kRing][kWave];                 // by lane: the next tasks of its list, task q in row q mod kRing
};

struct SchedCand {
    int pp, v, m, dp, tp;
    int state, n_rounds, depth, n_send;
    int st0, pool0;      // the candidate's first entries in the stage table and in the ring pool
    int64_t woff, poff, c;
};

template <int R>
__device__ __forceinline__ void scheduled_groups(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                                 const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                                 const SchedCand& xc, SchedLds& sm) {
    static_assert(R >= 2 && R <= kWave && (R & (R - 1)) == 0, "group sizes are powers of two from 2 to 64");
    constexpr int N = SchedLds::kRing, B = SchedLds::kBatch;
    const int lane = threadIdx.x, d = lane % R, g0 = lane - d;
    const int L = co.L;
    const int pp = xc.pp, v = xc.v, m = xc.m, dp = xc.dp, tp = xc.tp;
    const int64_t c = xc.c;
    bool grp = pp != 0;                                               // the group has a candidate in this pass
    bool act = grp && d < pp;
    // an invalid schedule: no strategy
    if (grp && xc.state == kSchedInvalid) {
        if (d == 0) { ev.status[c] = 1; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        grp = act = false;
    }
    const int32_t* w = ca.schedule_words + xc.woff;
    const uint64_t* ops = (const uint64_t*)ws.sched_ops + xc.woff;
    const int S = grp ? w[1] : 0, nparts = grp ? w[3] : 0, replicas = grp ? w[4] : 1;
    const int sb = 5 + pp + 1, tb = sb + 3 * S;
    const int ntask = grp ? w[5 + pp] : 0;
    const int t0 = act ? w[5 + d] : 0, t1 = act ? w[5 + d + 1] : 0;
    SchedStage* const st = sm.st + xc.st0;
    double* const pool = sm.pool + xc.pool0;
    double* const link_free = sm.link_free + 2 * xc.st0;

    // the partition: 0 = b0 < b1 < ... = L
    bool bad = false;
    for (int p = d; p < nparts; p += R) {
        int plo, phi;
        if (xc.poff >= 0) { plo = ca.part_pool[xc.poff + p]; phi = ca.part_pool[xc.poff + p + 1]; }
        else { plo = uniform_bound(p, L, nparts); phi = uniform_bound((p + 1), L, nparts); }
        if (phi <= plo || phi > L || (p == 0 && plo != 0) || (p == nparts - 1 && phi != L)) bad = true;
    }
    if (group_any(bad, R)) {
        if (grp && d == 0) { ev.status[c] = 1; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        grp = act = false;
    }

    // composed events of every stage's part, p2p events of the edges (lanes take the stages in turn)
    const int64_t tpdp = (int64_t)tp * dp;
    auto node_of = [&](int dev) -> int64_t {
        return tpdp >= cl.gpus_per_node ? dev : (int64_t)node_of_position(cl, dev, (int)tpdp);
    };
    const int64_t* row = ws.comb + (size_t)((v * kMaxPP + (pp > 0 ? pp - 1 : 0)) * (L + 1)) * kCombWords;
    const size_t vr = (size_t)v * (L + 1);
    auto bounds = [&](int part, int& lo, int& hi) {
        if (xc.poff >= 0) { lo = ca.part_pool[xc.poff + part]; hi = ca.part_pool[xc.poff + part + 1]; }
        else { lo = uniform_bound(part, L, nparts); hi = uniform_bound((part + 1), L, nparts); }
    };
    sm.dev_sum[0][lane] = 0; sm.dev_sum[1][lane] = 0; sm.dev_sum[2][lane] = 0;
    const int nS = grp ? S : 0;
    for (int k = d; k < nS; k += R) {
        const uint64_t info = ops[sb + 3 * k];
        const int prev = info_prev(info);
        int64_t PB = 0;
        if (prev >= 0) {
            // the activation that leaves the part of the stage before: entry of the layer after it
            const uint64_t pinfo = ops[sb + 3 * prev];
            int qlo, qhi;
            bounds(info_part(pinfo), qlo, qhi);
            const int inter = node_of(info_place(pinfo)) != node_of(info_place(info)) ? 1 : 0;
            PB = row[qhi * kCombWords + 4 + inter];
        }
        sm.own_p2p[xc.st0 + k] = PB;
        sm.queue[xc.st0 + k] = info_queue(info, 0) | info_queue(info, 1) << 8;
        link_free[k] = 0.0; link_free[S + k] = 0.0;
    }
    __syncthreads();
    int64_t share = 0;
    for (int k = d; k < nS; k += R) {
        const uint64_t info = ops[sb + 3 * k], cnt = ops[sb + 3 * k + 1];
        const int next = info_next(info);
        int lo, hi;
        bounds(info_part(info), lo, hi);
        const int64_t* eh = row + hi * kCombWords;
        const int64_t* el = row + lo * kCombWords;
        const int64_t FT = eh[0] - el[0], BT = eh[1] - el[1];
        const int64_t fcp = ws.pfc[vr + hi] - ws.pfc[vr + lo], bcp = ws.pbc[vr + hi] - ws.pbc[vr + lo];
        const int64_t PB = sm.own_p2p[xc.st0 + k], PF = next >= 0 ? sm.own_p2p[xc.st0 + next] : 0;
        share += FT + BT + PF + PB;
        const int64_t pf_task = cl.blocking == 1 ? PF : 0, pb_task = cl.blocking == 1 ? PB : 0;
        SchedStage s;
        s.dur_f = (double)(FT + pf_task);
        s.dur_b = (double)(BT + pb_task);
        // the forward edge into the stage carries PB, the backward edge PF; with queues on the links
        // the task's own transfer is what the loop needs: PF after a forward, PB after a backward
        s.add_f = cl.blocking == 0 ? (double)PB : cl.blocking == 2 ? (double)PF : 0.0;
        s.add_b = cl.blocking == 0 ? (double)PF : cl.blocking == 2 ? (double)PB : 0.0;
        st[k] = s;
        // busy sums: every listed task of the stage counts
        const int64_t nF = (int64_t)(cnt & 0xffff), nB = (int64_t)(cnt >> 16 & 0xffff);
        const int holder = g0 + info_place(info);
        atomicAdd(&sm.dev_sum[0][holder], (unsigned long long)(nF * fcp + nB * bcp));
        atomicAdd(&sm.dev_sum[1][holder], (unsigned long long)(nF * (FT - fcp + PF) + nB * (BT - bcp + PB)));
        atomicAdd(&sm.dev_sum[2][holder], (unsigned long long)(eh[3] - el[3]));
    }
    if (stage_out_of_range(grp ? share : 0, m, R)) {
        if (grp && d == 0) { ev.status[c] = 2; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        grp = act = false;
    }
    // lists that cannot be run to their ends
    if (grp && xc.state == kSchedStuck) {
        if (d == 0) { ev.status[c] = 1; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        grp = act = false;
    }
    __syncthreads();

    // the rounds.  A lane keeps the next tasks of its list in LDS: every kBatch rounds it asks for
    // those it has room for and stores them two rounds later, when they have arrived (a lane runs
    // at most one task per round, so it always has the next one there).
    const int n = act ? t1 : 0;                                       // the lane's tasks are [i, n)
    int i = act ? t0 : 0, req = i;
    {
        uint64_t first[N];
#pragma unroll
        for (int q = 0; q < N; q++) first[q] = i + q < n ? ops[tb + i + q] : 0;
#pragma unroll
        for (int q = 0; q < N; q++)
            if (i + q < n) sm.ops[(i + q) % N][lane] = first[q];
        req = i + N < n ? i + N : n;
    }
    uint64_t op = i < n ? sm.ops[i % N][lane] : ~0ull;                // (no round is 0xffff)
    uint64_t got[B];
    int n_got = 0;
    double own = 0.0;
    const int rounds = wave_max_i32(act ? xc.n_rounds : 0);
    auto loop = [&](auto links_tag) {
        constexpr bool LINKS = decltype(links_tag)::value;               // p2p_blocking = 2
        for (int round = 0; round < rounds; round++) {
            if ((round & (B - 1)) == 0) {
                // task q may take the place of task q - kRing once that one has been run
                n_got = 0;
#pragma unroll
                for (int q = 0; q < B; q++) {
                    const bool ask = req + q < n && req + q < i + N;
                    got[q] = ask ? ops[tb + req + q] : 0;
                    n_got += ask ? 1 : 0;
                }
            }
            if ((round & (B - 1)) == B / 2) {
#pragma unroll
                for (int q = 0; q < B; q++)
                    if (q < n_got) sm.ops[(req + q) % N][lane] = got[q];
                req += n_got;
                n_got = 0;
            }
            if (op_round(op) == round) {
                const int k = op_stage(op), kd = op_kind(op);
                const double* rec = &st[k].dur_f + 2 * kd;
                const double dur = rec[0], add = rec[1];
                const double e = pool[op_read_slot(op)];
                const uint64_t op_n = i + 1 < n ? sm.ops[(i + 1) % N][lane] : ~0ull;
                int queue = 0;
                double free_at = 0.0;
                if (LINKS) {
                    queue = sm.queue[xc.st0 + k] >> (8 * kd) & 0xff;
                    free_at = link_free[queue];
                }
                // one wait for all of them
                asm volatile("" : : "v"(dur), "v"(add), "v"(e), "v"(op_n), "v"(free_at));
                // with queues on the links the producer has stored the transfer's arrival time
                const double arrive = (op & kOpReads) ? (LINKS ? e : e + add) : 0.0;
                const double start = max_f64(arrive, own);
                own = start + dur;
                double seen = own;                                     // what the consuming task reads
                if (LINKS && (op & kOpFeeds)) {                        // the transfer queues on its link
                    seen = max_f64(own, free_at) + add;
                    link_free[queue] = seen;
                }
                if (op & kOpFeeds) pool[op_write_slot(op)] = seen;
                // bucketed all-reduce: a stage's gradients are complete in its last backward on the list
                if ((op & kOpLastBwd) && cl.bucket > 0) sm.lastb_start[xc.st0 + k] = start;
                i++;
                op = op_n;
            }
        }
    };
    if (cl.blocking == 2) loop(std::true_type{});
    else loop(std::false_type{});
    __syncthreads();

    // data-parallel modelling per device, as in explicit_candidate
    const int64_t ranks = (int64_t)dp * replicas;
    const int64_t endL = double_to_i64(own);
    const int64_t G = (int64_t)sm.dev_sum[2][lane];
    int64_t AR = 0, ar_last = endL, nar_dev = 0;                       // AR: busy time of the all-reduce events
    if (cl.bucket <= 0) {
        if (act && t1 > t0 && ranks > 1 && G > 0) { AR = allreduce_ns(cl, ranks, G); ar_last = endL + AR; nar_dev = 1; }
    } else if (act && ranks > 1) {
        const int64_t ar_cap = allreduce_ns(cl, ranks, cl.bucket);
        int64_t t_free = 0, acc = 0, ready = 0;
        for (int q = t0; q < t1; q++) {
            const uint64_t y = ops[tb + q];
            if (!(y & kOpLastBwd)) continue;
            const int k = op_stage(y);
            int lo, hi;
            bounds(info_part(ops[sb + 3 * k]), lo, hi);
            const int64_t startB = double_to_i64(sm.lastb_start[xc.st0 + k]), tot_hi = row[hi * kCombWords + 1];
            for (int l = hi - 1; l >= lo; l--) {
                ready = startB + (tot_hi - row[l * kCombWords + 1]);
                acc += row[(l + 1) * kCombWords + 3] - row[l * kCombWords + 3];
                const int64_t kb = (int64_t)udiv64_by((uint64_t)acc, (uint64_t)cl.bucket, cl.inv_bucket);
                if (kb > 0) {
                    const int64_t b0 = t_free > ready ? t_free : ready;
                    t_free = b0 + kb * ar_cap;
                    acc -= kb * cl.bucket;
                    AR += kb * ar_cap; nar_dev += kb;
                }
            }
        }
        if (acc > 0) {
            const int64_t b0 = t_free > ready ? t_free : ready, dd = allreduce_ns(cl, ranks, acc);
            t_free = b0 + dd;
            AR += dd; nar_dev++;
        }
        if (nar_dev > 0) ar_last = t_free;
    }
    const int64_t batch = group_max(act ? (ar_last > endL ? ar_last : endL) : 0, R);
    const int64_t nar = group_sum(act ? nar_dev : 0, R);
    if (act) {
        const int64_t base = ev.stage_pos[c];
        if (base >= 0) {
            const int64_t comp = (int64_t)sm.dev_sum[0][lane], comm = (int64_t)sm.dev_sum[1][lane];
            out.comp_busy[base + d] = comp;
            out.comm_busy[base + d] = comm + AR;
            if (out.util) out.util[base + d] = batch > 0 ? (double)comp / (double)batch : 0.0;
        }
        if (d == 0) {
            out.batch_ns[c] = batch;
            ev.num_events[c] = (int64_t)ntask + xc.n_send + nar;
        }
    }
    __syncthreads();
}

// One unit of work: the 64 / R consecutive candidates of the visiting order from pos0 on; those
// with an explicit schedule that has a program (or is invalid) are taken here.
template <int R>
__device__ __forceinline__ void scheduled_unit(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                               const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                               int64_t pos0, int64_t pos_end, SchedLds& sm) {
    constexpr int kGroups = kWave / R;
    const int lane = threadIdx.x, g = lane / R;
    // descriptors beyond the valid candidates were never written: the class table bounds them
    Desc ds{};
    if (pos0 + g < pos_end) ds = ws.desc[pos0 + g];
    if (!is_explicit(ds)) ds.meta = 0;
    int pp = ds.meta & 0xff;
    const int64_t id = ds.spare >> 32;
    SchedHdr h{kSchedTable, 0, 0, 0};
    if (pp != 0 && id < kSchedCap) h = ws.sched_hdr[id];
    if (h.state == kSchedTable) pp = 0;                                // k_simulate_explicit takes it
    const int S = pp != 0 && h.state != kSchedInvalid ? ca.schedule_words[ca.schedule_off[id] + 1] : 0;
    bool pending = pp != 0;
    // Passes: the pending candidates, in order, for as long as their stages and ring entries fit
    // (the first always does: at most 64 stages and kSchedMaxPool entries).
    for (int pass = 0; pass < kGroups && __builtin_amdgcn_ballot_w64(pending) != 0; pass++) {
        int stages = pending && lane % R == 0 ? S : 0, entries = pending && lane % R == 0 ? 2 * S * h.depth : 0;
        for (int sh = 1; sh < kWave; sh <<= 1) {
            const int a = __shfl_up(stages, sh, kWave), b = __shfl_up(entries, sh, kWave);
            if (lane >= sh) { stages += a; entries += b; }
        }
        const bool now = pending && stages <= SchedLds::kStages && entries <= kSchedWavePool;
        const SchedCand xc{now ? pp : 0, ds.meta >> 16, ds.m, ds.dp, (int)(uint32_t)ds.spare,
                           h.state, h.n_rounds, h.depth, h.n_send, now ? stages - S : 0, now ? entries - 2 * S * h.depth : 0,
                           now ? ca.schedule_off[id] : 0, ds.poff, ds.cand};
        if (__builtin_amdgcn_ballot_w64(now) == 0) break;               // cannot be
        scheduled_groups<R>(co, cl, ca, ws, ev, out, xc, sm);
        pending = pending && !now;
    }
}

// All classes in one launch, as k_simulate_virtual: class k of the visiting order holds the
// candidates of 64 >> k lanes and keeps those with an explicit schedule side by side; a block is
// one wavefront.
__global__ __launch_bounds__(kWave, 3) void k_simulate_scheduled(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                                 EventsDev ev, SimOut out) {
    __shared__ SchedLds sm;
    int64_t next = blockIdx.x;                    // this block's next unit, counted from the first unit of the current class
    auto one_class = [&](auto width_tag, int cls) {
        constexpr int R = decltype(width_tag)::value, kGroups = kWave / R;
        int64_t pos_lo, pos_end;
        explicit_range(ws, cls, pos_lo, pos_end);
        const int64_t units = (pos_end - pos_lo + kGroups - 1) / kGroups;
        for (; next < units; next += gridDim.x)
            scheduled_unit<R>(co, cl, ca, ws, ev, out, pos_lo + next * kGroups, pos_end, sm);
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

}  // namespace distsim
