// Timeline simulation: level-synchronous sweep of the pipeline recurrence of Algorithm 1.
#pragma once
#include "kernels_build.hpp"

namespace distsim {

struct SimOut {
    int64_t* batch_ns;
    int64_t* comp_busy;
    int64_t* comm_busy;
    double* util;       // may be null
};

__global__ __launch_bounds__(256) void k_sim_init(const int32_t* __restrict__ status, int64_t C,
                                                  int64_t* __restrict__ batch_ns) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c < C && status[c] != 0) batch_ns[c] = INT64_MAX;
}

// Lane (g, s) of a wave-item owns stage s of one candidate and keeps a single running value:
// the end time of the most recent stage-task on that device.  Tasks are visited in levels
// chosen such that every dependency of a level-l task lies in a lower level; for 1F1B and the
// asynchronous schedule, which shares its order (GPipe candidates are not swept, see gpipe_finish):
//   F(s,j): s + j        (j <= w_s)       B(s,j): 2 pp - 1 - s + 2 j
//           s + 2 j      (j >  w_s)       w_s = min(pp - 1 - s, m) warm-up forwards
// In that order the most recent task of the producing neighbour at the time a task runs is
// exactly its producer (forward: F(s-1,j) on the previous lane; backward: B(s+1,j) on the next
// lane), so the cross-stage operand is the neighbour lane's register, read with a DPP shift.
// Times are carried as doubles: every value is an integer below 2^53 (range guard at event
// generation), so fp64 add and max are exact and one instruction each.
//
// Which lanes run a forward / backward task at a level is precomputed 32 levels at a time as
// two per-lane bit patterns (bit 31 = first level of the chunk).  Adding a pattern to itself
// shifts it by one level and drops the current level's bit into the carry mask, which becomes
// the EXEC mask of the three fp64 instructions of the task: no per-level compares or selects.

// bits of the chunk-relative levels a..b (inclusive), bit 31 = level 0; empty when a > b or the
// range misses the chunk (64-bit shifts, so that shifting by 32 clears the word)
__device__ __forceinline__ uint32_t level_bits(int a, int b) {
    const int lo = a < 0 ? 0 : (a > 32 ? 32 : a);
    const int hi = b > 31 ? 31 : (b < -1 ? -1 : b);
    return (uint32_t)(0xffffffffull >> lo) & (uint32_t)(0xffffffffull << (31 - hi));
}

__device__ __forceinline__ uint32_t shl32(uint32_t x, int n) { return n >= 32 ? 0u : x << n; }

// Bitwise OR over the 64 lanes, returned as a wave-uniform value.
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) {
    int v = (int)x;
    v |= __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);     // quad_perm [1,0,3,2]
    v |= __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);     // quad_perm [2,3,0,1]
    v |= __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);    // row_half_mirror
    v |= __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);    // row_mirror
    return (uint32_t)(__builtin_amdgcn_readlane(v, 0) | __builtin_amdgcn_readlane(v, 16) |
                      __builtin_amdgcn_readlane(v, 32) | __builtin_amdgcn_readlane(v, 48));
}

// Operand of a level on which lanes of one parity run forwards and the others backwards:
// the previous lane's value for the forward lanes, the next lane's for the backward lanes,
// fetched with one ds_bpermute per 32-bit half (byte address = 4 * source lane).
// On odd levels the forward lanes are the odd stages and read stage s-1, the backward lanes
// are the even stages and read stage s+1: lanes 2k and 2k+1 read each other, which is one
// quad permutation.
__device__ __forceinline__ double from_pair_partner(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xf, 0xf, true);      // quad_perm [1,0,3,2]
    hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
// On even levels (past the warm-up) the forward lanes are the even stages and read stage s-1,
// the backward lanes are the odd stages and read stage s+1: no single DPP pattern, so the
// operand comes through one ds_bpermute per 32-bit half (byte address = 4 * source lane).
__device__ __forceinline__ double from_lanes(double x, int byte_addr) {
    const int lo = __builtin_amdgcn_ds_bpermute(byte_addr, __double2loint(x));
    const int hi = __builtin_amdgcn_ds_bpermute(byte_addr, __double2hiint(x));
    return __hiloint2double(hi, lo);
}

// Value held by the next / previous lane of the wavefront, the 64 lanes taken as a ring.
template <int CTRL>
__device__ __forceinline__ double dpp_move_f64(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
constexpr int kDppWaveRol1 = 0x134;   // lane i reads lane i+1, lane 63 reads lane 0
constexpr int kDppWaveRor1 = 0x13C;   // lane i reads lane i-1, lane 0 reads lane 63

// One level for the lanes whose pattern bit is set: own = max(own, nb + lat) + dur.
// Requires EXEC == all ones on entry (wave-uniform control flow, full wavefronts) and leaves
// it so.  The trailing s_nop keeps two wait states between the write of `own` and the DPP
// read that follows.  The *2 forms run the same level of two candidates' sweeps that share
// one shape, hence one pattern and one EXEC mask.
#define DISTSIM_STEP1(bits, o, t, lat, dur)                                    \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[p], %[k], %[p], %[p]\n\t"                        \
        "s_mov_b64 exec, %[k]\n\t"                                            \
        "v_add_f64 %[t0], %[t0], %[c0]\n\t"                                   \
        "v_max_f64 %[t0], %[t0], %[o0]\n\t"                                   \
        "v_add_f64 %[o0], %[t0], %[d0]\n\t"                                   \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o0] "+v"(o), [t0] "+v"(t), [p] "+v"(bits), [k] "=&s"(kmask)        \
        : [c0] "v"(lat), [d0] "v"(dur))

#define DISTSIM_STEP2(bits, oa, ta, lata, dura, ob, tb, latb, durb)            \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[p], %[k], %[p], %[p]\n\t"                        \
        "s_mov_b64 exec, %[k]\n\t"                                            \
        "v_add_f64 %[t0], %[t0], %[c0]\n\t"                                   \
        "v_add_f64 %[t1], %[t1], %[c1]\n\t"                                   \
        "v_max_f64 %[t0], %[t0], %[o0]\n\t"                                   \
        "v_max_f64 %[t1], %[t1], %[o1]\n\t"                                   \
        "v_add_f64 %[o0], %[t0], %[d0]\n\t"                                   \
        "v_add_f64 %[o1], %[t1], %[d1]\n\t"                                   \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o0] "+v"(oa), [t0] "+v"(ta), [o1] "+v"(ob), [t1] "+v"(tb), [p] "+v"(bits), [k] "=&s"(kmask) \
        : [c0] "v"(lata), [d0] "v"(dura), [c1] "v"(latb), [d1] "v"(durb))

// A level with forward lanes (operand from the previous lane) and backward lanes (operand from
// the next lane) in no particular arrangement: two masks, two task steps.
#define DISTSIM_STEPFB1(pf, pb, o, tl, tr, cl_, cr_, df, db)                   \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[pf_], %[kf], %[pf_], %[pf_]\n\t"                 \
        "v_add_co_u32_e64 %[pb_], %[kb], %[pb_], %[pb_]\n\t"                 \
        "s_mov_b64 exec, %[kf]\n\t"                                           \
        "v_add_f64 %[tl_], %[tl_], %[cl__]\n\t"                               \
        "v_max_f64 %[tl_], %[tl_], %[o_]\n\t"                                 \
        "v_add_f64 %[o_], %[tl_], %[df_]\n\t"                                 \
        "s_mov_b64 exec, %[kb]\n\t"                                           \
        "v_add_f64 %[tr_], %[tr_], %[cr__]\n\t"                               \
        "v_max_f64 %[tr_], %[tr_], %[o_]\n\t"                                 \
        "v_add_f64 %[o_], %[tr_], %[db_]\n\t"                                 \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o_] "+v"(o), [tl_] "+v"(tl), [tr_] "+v"(tr), [pf_] "+v"(pf), [pb_] "+v"(pb),   \
          [kf] "=&s"(kmask), [kb] "=&s"(kmask2)                               \
        : [cl__] "v"(cl_), [cr__] "v"(cr_), [df_] "v"(df), [db_] "v"(db))

// The same with masks that have already been taken from the patterns.
#define DISTSIM_APPLYFB(o, tl, tr, cl_, cr_, df, db)                           \
    asm volatile(                                                              \
        "s_mov_b64 exec, %[kf]\n\t"                                           \
        "v_add_f64 %[tl_], %[tl_], %[cl__]\n\t"                               \
        "v_max_f64 %[tl_], %[tl_], %[o_]\n\t"                                 \
        "v_add_f64 %[o_], %[tl_], %[df_]\n\t"                                 \
        "s_mov_b64 exec, %[kb]\n\t"                                           \
        "v_add_f64 %[tr_], %[tr_], %[cr__]\n\t"                               \
        "v_max_f64 %[tr_], %[tr_], %[o_]\n\t"                                 \
        "v_add_f64 %[o_], %[tr_], %[db_]\n\t"                                 \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o_] "+v"(o), [tl_] "+v"(tl), [tr_] "+v"(tr)                        \
        : [kf] "s"(kmask), [kb] "s"(kmask2), [cl__] "v"(cl_), [cr__] "v"(cr_), [df_] "v"(df), [db_] "v"(db))

// One level of the sweep with queues on the links (p2p_blocking = 2), for the lanes whose pattern bit
// is set: the task starts at max(own, arrival of the neighbour's latest send) -- `gate` is 0 for a
// lane that has that neighbour and -inf for one that has not --, and its own send leaves when the
// task has ended and the link is free: own = max(own, arr + gate) + dur; link = max(own, link) + send.
#define DISTSIM_LSTEP(bits, o, t, link, gate, dur, send)                       \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[p], %[k], %[p], %[p]\n\t"                        \
        "s_mov_b64 exec, %[k]\n\t"                                            \
        "v_add_f64 %[t0], %[t0], %[g0]\n\t"                                   \
        "v_max_f64 %[t0], %[t0], %[o0]\n\t"                                   \
        "v_add_f64 %[o0], %[t0], %[d0]\n\t"                                   \
        "v_max_f64 %[t0], %[o0], %[l0]\n\t"                                   \
        "v_add_f64 %[l0], %[t0], %[s0]\n\t"                                   \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o0] "+v"(o), [t0] "+v"(t), [l0] "+v"(link), [p] "+v"(bits), [k] "=&s"(kmask) \
        : [g0] "v"(gate), [d0] "v"(dur), [s0] "v"(send))

// Level windows of a lane that holds stage s, expressed on x = level - s:
//   forward  x in [0, f1hi]  and  even x in [f2lo, f2hi]
//   backward x in [blo, bhi], every second x
struct LevelWindows {
    int f1hi, f2lo = 1, f2hi = 0, blo, bhi;
    __device__ __forceinline__ LevelWindows(int m, int pp, int s) {
        int wq = pp - 1 - s; if (wq > m) wq = m;
        f1hi = wq < m - 1 ? wq : m - 1;
        f2lo = 2 * wq + 2; f2hi = 2 * m - 2;
        blo = 2 * pp - 1 - 2 * s; bhi = blo + 2 * m - 2;
    }
};

// Per-lane state of one candidate's sweep.
struct Sweep {
    double own;            // end of the most recent task on this device
    double pfL, pbR;       // p2p latency on the incoming forward / backward edge, -inf = no edge
    double Fd, Bd;         // duration of a forward / backward stage-task
};

// One wavefront per workgroup: a wavefront's slot and LDS are free again when its own items are done,
// not when the slowest of four is (measured against 256 threads: span -1.5 %, gpt96 -2.4 %).
constexpr int kSimBlock = 64;
// The DISTSIM_STEP* macros set EXEC themselves and put it back to all ones: every kernel that uses
// them must run whole 64-lane wavefronts and call them from wave-uniform control flow only.
static_assert(kSimBlock % kWave == 0, "the sweep kernels need whole wavefronts");

// What only the epilogue of an item needs waits here during the sweep, one slot per lane of the
// workgroup and per item of a lockstep pair (one block, so that one address register serves).
struct Park {
    int64_t comp[2][kSimBlock];        // computation per micro-batch
    int64_t comm[2][kSimBlock];        // communication per micro-batch
    int64_t ar[2][kSimBlock];          // single trailing all-reduce
    int32_t cand[2][kSimBlock];
    int32_t dp[2][kSimBlock];
    int32_t misc[2][kSimBlock];        // layer bounds, flags, variant
};

// GPipe without a sweep.  The events of a stage are the same for every micro-batch (Sec. 4.3: the
// stage's event list is built once and replayed), so under GPipe the m forwards, and then the m
// backwards, pass the stages as identical jobs pass the machines of a flow shop, and the recurrence
// start = max(end of the device's previous task, end of the producer + p2p) solves exactly:
//   end F(s, j) = sum_{i<=s} (F_i + pf_i) + j max_{i<=s} F_i
// (induction on s and j: of the two operands of the max, the producer's wins when an earlier stage
// is the longest, the device's own previous task when stage s is), and for the backwards, which
// the last stage starts when its last forward has ended at R = end F(pp-1, m-1),
//   end B(s, j) = R + sum_{i>=s} (B_i + pb_i) + j max_{i>=s} B_i
// (the same induction from the last stage down; a path that starts at the end of an earlier
// stage's forwards instead is never longer, since R, the sums and the maxima only grow towards
// the last stage).  F_i, B_i: duration of a stage-task on its device, the send included when the
// sender is occupied by it; pf_i, pb_i: latency of the edge into stage i, zero for the first
// stage of either direction.  LINKS (sends queue on their link, one transfer at a time): a link is
// one more machine of the shop, between its two stages, so its transfer time also enters the two
// maxima.  What the epilogue needs is the end of each stage's last backward:
// one reduction over the candidate's lanes and two suffix scans, in exact fp64 (every partial
// sum is an integer below 2^53 by the range check).  Lanes with on[u] unset contribute nothing.
template <int U, bool LINKS = false>
__device__ __forceinline__ void gpipe_finish(const Sweep (&sw)[U], const bool (&on)[U], const int (&m)[U],
                                             int s, int width, int lane, double (&fin)[U]) {
    double fs[U], fm[U], T[U], M[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
        // an edge that does not exist carries -inf
        const double eF = max_f64(sw[u].pfL, 0.0), eB = max_f64(sw[u].pbR, 0.0);
        fs[u] = on[u] ? sw[u].Fd + eF : 0.0;
        fm[u] = on[u] ? (LINKS ? max_f64(sw[u].Fd, eF) : sw[u].Fd) : 0.0;
        T[u] = on[u] ? sw[u].Bd + eB : 0.0;
        M[u] = on[u] ? (LINKS ? max_f64(sw[u].Bd, eB) : sw[u].Bd) : 0.0;
        fs[u] = group_sum_f64(fs[u], width);
        fm[u] = group_max_f64(fm[u], width);
    }
    // inclusive suffix sum / suffix maximum over the candidate's lanes; a lane whose partner would
    // lie outside the candidate reads itself, which leaves a maximum as it is
    for (int d = 1; d < width; d <<= 1) {
        const bool ok = s + d < width;
        const int adr = (ok ? lane + d : lane) * 4;
#pragma unroll
        for (int u = 0; u < U; u++) {
            const double t = from_lanes(T[u], adr), x = from_lanes(M[u], adr);
            T[u] += ok ? t : 0.0;
            M[u] = max_f64(M[u], x);
        }
    }
#pragma unroll
    for (int u = 0; u < U; u++) fin[u] = fs[u] + T[u] + (double)(m[u] - 1) * (fm[u] + M[u]);
}

// Simulates U wave-items at once.  For U = 2 the two items must have the same shape in every
// lane (pp, m, schedule): then they share patterns, masks and control flow.  GPipe candidates take
// no part in the sweep: their end times have a closed form (gpipe_finish).  GPIPE_PAIR: the two
// items hold nothing but GPipe candidates, of any shapes; the caller has checked that.
template <int U, bool LINKS = false, bool GPIPE_PAIR = false>
__device__ __forceinline__ void simulate_items(const ClusterDev& cl, const CandDev& ca, const Workspace& ws,
                                               const EventsDev& ev, const SimOut& out, int L, int64_t w0,
                                               int sh, const Desc (&d)[U], int lane,
                                               Park& park) {
    const double ninf = -__builtin_huge_val();
    const int slot = threadIdx.x;
    const int width = 1 << sh;
    const int s = lane & (width - 1);
    // shape: shared by the U items, except in a GPipe pair, where each item has its own
    int ppv[U], mv[U];
    bool actv[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
        const Desc& ds = d[GPIPE_PAIR ? u : 0];
        ppv[u] = ds.meta & 0xff;
        actv[u] = s < ppv[u];
        mv[u] = actv[u] ? ds.m : 0;
    }
    const int pp = ppv[0], sched = (d[0].meta >> 8) & 0xff, m = mv[0];
    const bool act = actv[0];

    Sweep sw[U];
    double sendF[U], sendB[U];      // LINKS: duration of this stage's outgoing forward / backward send
#pragma unroll
    for (int u = 0; u < U; u++) {
        const int v = d[u].meta >> 16, dp = d[u].meta ? d[u].dp : 1;
        const int64_t c = d[u].cand;
        // the stage's composed events, regenerated from the layer-event tables
        int lo = 0, hi = 0;
        if (actv[u]) {
            if (d[u].poff >= 0) { lo = ca.part_pool[d[u].poff + s]; hi = ca.part_pool[d[u].poff + s + 1]; }
            else { lo = uniform_bound(s, L, ppv[u]); hi = uniform_bound((s + 1), L, ppv[u]); }
        }
        StageSums r;
        const int drop = stage_sums(cl, ws, L, width, s, ppv[u], v, d[u].m, dp, (int)d[u].spare, lo, hi, r);
        if (drop && actv[u] && s == 0) { ev.status[c] = drop; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
        // gradient bytes to reduce over dp > 1 ranks; the asynchronous schedule has no such event
        const bool has_ar = actv[u] && dp > 1 && r.G > 0 && sched != 2;
        // p2p on the incoming edges (the neighbours' outgoing events): latency of the edge, or,
        // when the sender is occupied by it, part of the sender's task; -inf = no edge
        const int64_t pf_task = cl.blocking == 1 ? r.PF : 0, pb_task = cl.blocking == 1 ? r.PB : 0;
        sw[u].own = 0.0;
        sw[u].Fd = (double)(r.FT + pf_task);
        sw[u].Bd = (double)(r.BT + pb_task);
        sw[u].pfL = from_prev_lane((double)(r.PF - pf_task));
        sw[u].pbR = from_next_lane((double)(r.PB - pb_task));
        sendF[u] = (double)r.PF; sendB[u] = (double)r.PB;
        if (!(actv[u] && s > 0)) sw[u].pfL = ninf;
        if (!(actv[u] && s + 1 < ppv[u])) sw[u].pbR = ninf;
        // what only the epilogue needs waits in LDS
        park.comp[u][slot] = r.CP;                                         // computation per micro-batch
        park.comm[u][slot] = r.FT + r.BT - r.CP + r.PF + r.PB;             // communication per micro-batch
        park.ar[u][slot] = (cl.bucket > 0 || !has_ar) ? 0 : allreduce_ns_by(cl, dp, r.G, r.inv_ar);  // single trailing all-reduce
        park.cand[u][slot] = (int32_t)c;
        park.dp[u][slot] = dp;
        park.misc[u][slot] = lo | (hi << 8) | ((int)has_ar << 16) | ((drop ? 1 : 0) << 17) | (v << 18);
    }

    if constexpr (LINKS) {
        const LevelWindows lw(m, pp, s);
        const int f1hi = lw.f1hi, f2lo = lw.f2lo, f2hi = lw.f2hi, blo = lw.blo, bhi = lw.bhi;
        // Sends queue on their link (p2p_blocking = 2): every lane keeps the arrival time of its
        // latest forward send and of its latest backward send; a send starts when its task has
        // ended and the link is free, and the neighbour reads the arrival time instead of the end
        // of the task.  Plain per-level form of the sweep, one item at a time.
        static_assert(U == 1, "the serialised sweep takes one item at a time");
        const bool gpipe = act && sched == 0;       // closed form below
        const bool swept = act && sched != 0;
        const int nlev = wave_max_i32(swept ? 2 * (m + pp - 1) : 0);
        // a lane without that neighbour never looks at what the lane beside it sends (another
        // candidate's stage); the link time of a lane without a receiver is never looked at either
        const double gateL = act && s > 0 ? 0.0 : ninf, gateR = act && s + 1 < pp ? 0.0 : ninf;
        double own = 0.0, linkF = 0.0, linkB = 0.0;
        // The warm-up forwards in closed form, as in the sweep without queues (below): with a link that
        // carries one transfer at a time the shop has one more machine between two stages, the link.
        // end F(s, j) = (sum + j max) over the stages up to s and the links in front of s; the arrival
        // of stage s's latest send adds its own link to both.
        {
            const double before = from_prev_lane(sendF[0]);
            const double inL = swept && s > 0 ? before : 0.0;              // transfer on the link into this stage
            double acc = swept ? sw[0].Fd + inL : 0.0, top = swept ? max_f64(sw[0].Fd, inL) : 0.0;
            for (int dd = 1; dd < width; dd <<= 1) {
                const bool ok = s >= dd;
                const int adr = (ok ? lane - dd : lane) * 4;
                const double t = from_lanes(acc, adr), x = from_lanes(top, adr);
                acc += ok ? t : 0.0;
                top = max_f64(top, x);
            }
            if (swept) {
                own = __fma_rn((double)f1hi, top, acc);
                linkF = __fma_rn((double)f1hi, max_f64(top, sendF[0]), acc + sendF[0]);
            }
        }
        const int first = -wave_max_i32(swept ? -(s + blo) : -(1 << 30));      // level of the first backward
        uint64_t kmask;
        for (int l0 = first; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;
            uint32_t PFb = level_bits(f2lo - x0, f2hi - x0) & even_x;               // the forwards behind the warm-up
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;
            if (!swept) { PFb = 0; PBb = 0; }
            const bool anyF = wave_or_u32(PFb) != 0, anyB = wave_or_u32(PBb) != 0;
            const int kend = nlev - l0 < 32 ? nlev - l0 : 32;
            // a lane runs at most one task per level, and a level's tasks read only what the level
            // before left: the backward step may follow the forward step, which changes neither the
            // backward lanes' end times nor any backward link
            for (int k = 0; k < kend; k++) {
                if (anyF) {
                    double arrL = from_prev_lane(linkF);
                    DISTSIM_LSTEP(PFb, own, arrL, linkF, gateL, sw[0].Fd, sendF[0]);
                }
                if (anyB) {
                    double arrR = from_next_lane(linkB);
                    DISTSIM_LSTEP(PBb, own, arrR, linkB, gateR, sw[0].Bd, sendB[0]);
                }
            }
            (void)kmask;
        }
        sw[0].own = own;
        if (__builtin_amdgcn_ballot_w64(gpipe) != 0) {
            const bool on[1] = {gpipe};
            const int mg[1] = {m};
            double fin[1];
            gpipe_finish<1, true>(sw, on, mg, s, width, lane, fin);
            if (gpipe) sw[0].own = fin[0];
        }
    } else if constexpr (GPIPE_PAIR) {
        double fin[U];
        gpipe_finish<U>(sw, actv, mv, s, width, lane, fin);
#pragma unroll
        for (int u = 0; u < U; u++) sw[u].own = fin[u];
    } else {
        const LevelWindows lw(m, pp, s);
        const bool gpipe = act && sched == 0;       // closed form below
        const bool swept = act && sched != 0;
        // GPipe lanes first: the sweep below never touches them (their patterns are empty)
        if (__builtin_amdgcn_ballot_w64(gpipe) != 0) {
            bool on[U];
            int mg[U];
            double fin[U];
#pragma unroll
            for (int u = 0; u < U; u++) { on[u] = gpipe; mg[u] = m; }
            gpipe_finish<U>(sw, on, mg, s, width, lane, fin);
#pragma unroll
            for (int u = 0; u < U; u++) if (gpipe) sw[u].own = fin[u];
        }
        const int f1hi = lw.f1hi, f2lo = lw.f2lo, f2hi = lw.f2hi, blo = lw.blo, bhi = lw.bhi;
        // The warm-up without a sweep.  The forwards in front of a stage's first backward, F(s, j) with
        // j <= f1hi, depend on F(s-1, j) and F(s, j-1) only, and both lie in the warm-up as well (an
        // earlier stage warms up at least as long): on that set the recurrence is the flow shop of
        // gpipe_finish, end F(s, j) = sum_{i<=s} (F_i + pf_i) + j max_{i<=s} F_i.  Every lane starts the
        // sweep with the end of its last warm-up forward, which is the state the level sweep reaches
        // at the candidate's first backward (level pp); the levels in front of it are not visited.
        // One prefix sum and one prefix maximum over the candidate's lanes, exact in fp64.
        if (__builtin_amdgcn_ballot_w64(swept) != 0) {
            double acc[U], top[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                acc[u] = swept ? sw[u].Fd + max_f64(sw[u].pfL, 0.0) : 0.0;     // an edge that does not exist carries -inf
                top[u] = swept ? sw[u].Fd : 0.0;
            }
            for (int dd = 1; dd < width; dd <<= 1) {
                const bool ok = s >= dd;
                const int adr = (ok ? lane - dd : lane) * 4;
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const double t = from_lanes(acc[u], adr), x = from_lanes(top[u], adr);
                    acc[u] += ok ? t : 0.0;
                    top[u] = max_f64(top[u], x);
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) if (swept) sw[u].own = __fma_rn((double)f1hi, top[u], acc[u]);
        }
        // Levels at which some lane of the wavefront has a task left: forwards behind the warm-up up to
        // gLastF, backwards from gFirstB (the first level of the sweep) to gLastB (its last).
        const int gLastF = wave_max_i32(swept && f2lo <= f2hi ? s + f2hi : -1);
        const int gFirstB = -wave_max_i32(swept ? -(s + blo) : -(1 << 30));
        const int gLastB = wave_max_i32(swept ? s + bhi : -1);
        const int nlev = gLastB + 1;

        // 1F1B past its warm-up runs forwards on even x and backwards on odd x.  When every
        // candidate of the wavefront is 1F1B with one pp, a level that has both kinds therefore
        // splits the lanes by parity, and one merged operand (previous lane for the forward
        // lanes, next lane for the backward lanes) feeds a single task step.
        const int ppu = wave_max_i32(swept ? pp : 0);
        const bool par_ok = width >= 2 && __builtin_amdgcn_ballot_w64(swept && pp != ppu) == 0;
        const bool even_s = (s & 1) == 0;
        const int adrE = (even_s ? lane - 1 : lane + 1) * 4;

        for (int l0 = gFirstB; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;       // levels with even x
            uint32_t PFb = level_bits(f2lo - x0, f2hi - x0) & even_x;            // the forwards behind the warm-up
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;                   // x - blo even
            if (!swept) { PFb = 0; PBb = 0; }
            // chunk-relative level ranges in which a lane may have a forward / a backward task
            const bool anyF = gLastF >= l0, anyB = gFirstB < l0 + 32;
            const int firstF = anyF ? 0 : 64, lastF = anyF ? (gLastF - l0 < 31 ? gLastF - l0 : 31) : -1;
            const int firstB = anyB ? (gFirstB > l0 ? gFirstB - l0 : 0) : 64;
            const int lastB = anyB ? (gLastB - l0 < 31 ? gLastB - l0 : 31) : -1;
            const int endk = (lastF > lastB ? lastF : lastB) + 1;
            int k = firstF < firstB ? firstF : firstB;
            PFb = shl32(PFb, k); PBb = shl32(PBb, k);            // skip the idle levels in front
            uint64_t kmask, kmask2;
            while (k < endk) {
                const bool inF = k >= firstF && k <= lastF, inB = k >= firstB && k <= lastB;
                int e = endk;                                     // next level at which the mix changes
                if (firstF > k && firstF < e) e = firstF;
                if (firstB > k && firstB < e) e = firstB;
                if (lastF + 1 > k && lastF + 1 < e) e = lastF + 1;
                if (lastB + 1 > k && lastB + 1 < e) e = lastB + 1;
                const int len = e - k;
                if (inF && inB && par_ok) {
                    // roles by parity: on even levels the even stages run forwards, on odd levels
                    // the odd stages do
                    double latE[U], durE[U], latO[U], durO[U];
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        latE[u] = even_s ? sw[u].pfL : sw[u].pbR; durE[u] = even_s ? sw[u].Fd : sw[u].Bd;
                        latO[u] = even_s ? sw[u].pbR : sw[u].pfL; durO[u] = even_s ? sw[u].Bd : sw[u].Fd;
                    }
                    uint32_t Pc = PFb | PBb;
                    // straight-line (odd level, even level) pairs, so that both kinds of level keep
                    // their state in the same registers; a leading even and a trailing odd level apart
                    auto odd_level = [&]() {
                        if constexpr (U == 1) {
                            double nb = from_pair_partner(sw[0].own);
                            DISTSIM_STEP1(Pc, sw[0].own, nb, latO[0], durO[0]);
                        } else {
                            double na = from_pair_partner(sw[0].own), nb = from_pair_partner(sw[U - 1].own);
                            DISTSIM_STEP2(Pc, sw[0].own, na, latO[0], durO[0], sw[U - 1].own, nb, latO[U - 1], durO[U - 1]);
                        }
                    };
                    auto even_level = [&]() {
                        if constexpr (U == 1) {
                            double nb = from_lanes(sw[0].own, adrE);
                            DISTSIM_STEP1(Pc, sw[0].own, nb, latE[0], durE[0]);
                        } else {
                            double na = from_lanes(sw[0].own, adrE), nb = from_lanes(sw[U - 1].own, adrE);
                            DISTSIM_STEP2(Pc, sw[0].own, na, latE[0], durE[0], sw[U - 1].own, nb, latE[U - 1], durE[U - 1]);
                        }
                    };
                    int j = 0;
                    if (((l0 + k) & 1) == 0) { even_level(); j = 1; }
                    for (; j + 1 < len; j += 2) { odd_level(); even_level(); }
                    if (j < len) odd_level();
                    PFb = shl32(PFb, len); PBb = shl32(PBb, len);
                } else if (inF && inB) {
                    for (int j = 0; j < len; j++) {
                        double fl = from_prev_lane(sw[0].own), fr = from_next_lane(sw[0].own);
                        DISTSIM_STEPFB1(PFb, PBb, sw[0].own, fl, fr, sw[0].pfL, sw[0].pbR, sw[0].Fd, sw[0].Bd);
                        if constexpr (U == 2) {
                            double gl = from_prev_lane(sw[U - 1].own), gr = from_next_lane(sw[U - 1].own);
                            DISTSIM_APPLYFB(sw[U - 1].own, gl, gr, sw[U - 1].pfL, sw[U - 1].pbR, sw[U - 1].Fd, sw[U - 1].Bd);
                        }
                    }
                } else if (inF) {
                    for (int j = 0; j < len; j++) {
                        if constexpr (U == 1) {
                            double fl = from_prev_lane(sw[0].own);
                            DISTSIM_STEP1(PFb, sw[0].own, fl, sw[0].pfL, sw[0].Fd);
                        } else {
                            double fl = from_prev_lane(sw[0].own), gl = from_prev_lane(sw[U - 1].own);
                            DISTSIM_STEP2(PFb, sw[0].own, fl, sw[0].pfL, sw[0].Fd, sw[U - 1].own, gl, sw[U - 1].pfL, sw[U - 1].Fd);
                        }
                    }
                    PBb = shl32(PBb, len);
                } else if (inB) {
                    bool packed = false;
                    if constexpr (U == 2) {
                        // The cool-down of two items in the lanes of one.  B(s, j) runs at level
                        // 2 pp - 1 - s + 2 j: a lane has a backward only when level + s is odd, so at any
                        // level every second lane idles.  The second item is rotated by one lane inside
                        // each candidate's lanes (lane s holds its stage s - 1, the last stage wraps to
                        // lane 0; width is even): its stage in lane s runs when level + s is even.  Each
                        // lane then alternates between the two items level by level, and with the two
                        // items' registers mixed by lane parity once (set O: what a lane runs on odd
                        // levels, set E: on even levels) one task step serves both items: the operand of
                        // an odd level is set E's end time of the next lane (the same item's next stage:
                        // first item for even lanes, second for odd lanes), and the other way round.  A
                        // lane without a next stage reads some value and adds -inf.  Six VALU
                        // instructions per level for the pair instead of eleven.  For candidates that
                        // fill the wavefront (64 lanes): the ring of lanes is then the DPP wave rotation.
                        packed = width == kWave && len >= 8;
                        if (packed) {
                            // mixed in place: item 0's registers become set O, item 1's set E
                            {
                                const double rOwn = dpp_move_f64<kDppWaveRor1>(sw[1].own), rLat = dpp_move_f64<kDppWaveRor1>(sw[1].pbR),
                                             rDur = dpp_move_f64<kDppWaveRor1>(sw[1].Bd);
                                sw[1].own = even_s ? rOwn : sw[0].own; sw[1].pbR = even_s ? rLat : sw[0].pbR; sw[1].Bd = even_s ? rDur : sw[0].Bd;
                                sw[0].own = even_s ? sw[0].own : rOwn; sw[0].pbR = even_s ? sw[0].pbR : rLat; sw[0].Bd = even_s ? sw[0].Bd : rDur;
                            }
                            uint32_t PM = PBb | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)PBb, kDppWaveRor1, 0xf, 0xf, true);
                            int j = 0;
                            if (((l0 + k) & 1) == 0) {
                                double nb = dpp_move_f64<kDppWaveRol1>(sw[0].own);
                                DISTSIM_STEP1(PM, sw[1].own, nb, sw[1].pbR, sw[1].Bd);
                                j = 1;
                            }
                            for (; j + 1 < len; j += 2) {
                                double na = dpp_move_f64<kDppWaveRol1>(sw[1].own);
                                DISTSIM_STEP1(PM, sw[0].own, na, sw[0].pbR, sw[0].Bd);
                                double nb = dpp_move_f64<kDppWaveRol1>(sw[0].own);
                                DISTSIM_STEP1(PM, sw[1].own, nb, sw[1].pbR, sw[1].Bd);
                            }
                            if (j < len) {
                                double na = dpp_move_f64<kDppWaveRol1>(sw[1].own);
                                DISTSIM_STEP1(PM, sw[0].own, na, sw[0].pbR, sw[0].Bd);
                            }
                            // and apart again
                            {
                                const double aOwn = even_s ? sw[0].own : sw[1].own, aLat = even_s ? sw[0].pbR : sw[1].pbR,
                                             aDur = even_s ? sw[0].Bd : sw[1].Bd;
                                const double bOwn = even_s ? sw[1].own : sw[0].own, bLat = even_s ? sw[1].pbR : sw[0].pbR,
                                             bDur = even_s ? sw[1].Bd : sw[0].Bd;
                                sw[0].own = aOwn; sw[0].pbR = aLat; sw[0].Bd = aDur;
                                sw[1].own = dpp_move_f64<kDppWaveRol1>(bOwn); sw[1].pbR = dpp_move_f64<kDppWaveRol1>(bLat);
                                sw[1].Bd = dpp_move_f64<kDppWaveRol1>(bDur);
                            }
                            PBb = shl32(PBb, len);
                        }
                    }
                    if (!packed)
                    for (int j = 0; j < len; j++) {
                        if constexpr (U == 1) {
                            double fr = from_next_lane(sw[0].own);
                            DISTSIM_STEP1(PBb, sw[0].own, fr, sw[0].pbR, sw[0].Bd);
                        } else {
                            double fr = from_next_lane(sw[0].own), gr = from_next_lane(sw[U - 1].own);
                            DISTSIM_STEP2(PBb, sw[0].own, fr, sw[0].pbR, sw[0].Bd, sw[U - 1].own, gr, sw[U - 1].pbR, sw[U - 1].Bd);
                        }
                    }
                    PFb = shl32(PFb, len);
                } else {
                    PFb = shl32(PFb, len); PBb = shl32(PBb, len);
                }
                k = e;
            }
            (void)kmask; (void)kmask2;
        }
    }

#pragma unroll
    for (int u = 0; u < U; u++) {
        // data-parallel modelling: gradient all-reduce after (or overlapped with) the last backward
        const int64_t AR = park.ar[u][slot];
        const int misc = park.misc[u][slot];
        const bool has_ar = (misc >> 16) & 1, dropped = (misc >> 17) & 1;
        const bool live = actv[u] && !dropped;      // lanes outside a candidate and dropped candidates have zero rows
        int64_t ar_busy = AR, nar = has_ar ? 1 : 0;
        int64_t batch = 0;
        double batch_d = 0.0;
        // One trailing event: the end of the batch can stay in fp64.  Sums below 2^52 are exact (both
        // terms are integers); a wavefront in which some lane's sum is not takes the integer path.
        bool in_f64 = cl.bucket <= 0;
        if (in_f64) {
            batch_d = group_max_f64(live ? sw[u].own + (double)AR : 0.0, width);
            in_f64 = __builtin_amdgcn_ballot_w64(!(batch_d < 4503599627370496.0)) == 0;
            batch = small_double_to_i64(batch_d);
        }
        if (!in_f64) {
            const int64_t endB = (int64_t)sw[u].own;
            int64_t finish = endB + AR;
            if (has_ar && cl.bucket > 0) {
                // Bucketed gradient all-reduce behind the last micro-batch's backward: layer l (taken from
                // hi - 1 down to lo) is ready at r_l = start of that backward + its events from hi - 1
                // down to l, the open bucket then holds the bytes of the layers l..hi-1 modulo the bucket
                // size, every full bucket is issued at once and the events queue on the device's
                // communication stream, t <- max(t, r_l) + (buckets issued at l) * ar_cap; the rest goes
                // after the stage's first layer.  Unrolled, that max-plus chain is
                //   t = max over l of  r_l + (events issued at the layers l, l-1, ..., lo)
                // and the number of full buckets issued by the layers above l is floor(bytes above l /
                // bucket size), so every term stands on its own: no chain through the layers, and their
                // table reads are independent.  (A layer that issues nothing adds a term that the next
                // issuing layer below it, or the end of the backward itself, dominates.)
                const int lo = misc & 0xff, hi = (misc >> 8) & 0xff, v = misc >> 18, dp = park.dp[u][slot];
                // per layer boundary: backward time of the layers below it (word 1), their gradient bytes (word 3)
                const int64_t* row = ws.comb + (size_t)((v * kMaxPP + ppv[u] - 1) * (L + 1)) * kCombWords;
                const int64_t startB = endB - (int64_t)sw[u].Bd;
                const int64_t tot_hi = row[hi * kCombWords + 1], g_hi = row[hi * kCombWords + 3];
                const double inv_ar = __longlong_as_double(row[5]);      // 1 / (dp * beta) of the row's all-reduce group
                const int64_t ar_cap = allreduce_ns_by(cl, dp, cl.bucket, inv_ar);
                const int64_t G = g_hi - row[lo * kCombWords + 3];
                const int64_t full = (int64_t)udiv64_by((uint64_t)G, (uint64_t)cl.bucket, cl.inv_bucket);
                const int64_t rest = G - full * cl.bucket;
                const int64_t dlast = rest > 0 ? allreduce_ns_by(cl, dp, rest, inv_ar) : 0;
                ar_busy = full * ar_cap + dlast;
                nar = full + (rest > 0 ? 1 : 0);
                const int64_t all = startB + tot_hi + ar_busy;          // r_l + events from l down = all - (time below l) - (events above l)
                int64_t t = endB;
                // four layers at a time, their table entries requested together (at clamped, always valid
                // addresses): a trip to memory per four layers instead of one per layer
                constexpr int kBatch = 4;
                for (int l0 = lo; l0 < hi; l0 += kBatch) {
                    int64_t gb[kBatch], tb[kBatch];
#pragma unroll
                    for (int i = 0; i < kBatch; i++) {
                        const int l = l0 + i < hi ? l0 + i : hi - 1;
                        gb[i] = row[(l + 1) * kCombWords + 3];
                        tb[i] = row[l * kCombWords + 1];
                    }
#pragma unroll
                    for (int i = 0; i < kBatch; i++) {
                        const int64_t above = (int64_t)udiv64_by((uint64_t)(g_hi - gb[i]), (uint64_t)cl.bucket, cl.inv_bucket);
                        const int64_t term = all - tb[i] - above * ar_cap;      // a clamped entry repeats the last layer's term
                        t = term > t ? term : t;
                    }
                }
                finish = t;
            }
            batch = group_max(live ? finish : 0, width);
            batch_d = (double)batch;
        }
        // one event per stage that has one, or the stages' bucket counts
        nar = cl.bucket > 0 ? group_sum(nar, width) : group_count(has_ar, width);
        const int64_t comp = live ? (int64_t)mv[u] * park.comp[u][slot] : 0;
        const int64_t comm = live ? (int64_t)mv[u] * park.comm[u][slot] + ar_busy : 0;
        const int64_t i = (w0 + u) * kWave + lane;
        // the rows are written once and not read again by the library: streaming stores
        __builtin_nontemporal_store(comp, &out.comp_busy[i]);
        __builtin_nontemporal_store(comm, &out.comm_busy[i]);
        if (out.util) __builtin_nontemporal_store(batch > 0 ? (double)comp / batch_d : 0.0, &out.util[i]);
        if (live && s == 0) {
            const int64_t cc = park.cand[u][slot];
            out.batch_ns[cc] = batch;
            // m (2 pp + 2 (pp - 1)) stage-tasks and p2p events: below 2^24 for m <= 2^16, pp <= 64
            ev.num_events[cc] = (int64_t)(2 * mv[u] * (2 * ppv[u] - 1)) + nar;
        }
    }
}

// Two launches share the wave-items.  In every class the leading items that hold only GPipe
// candidates (hdr[H_GPIPE_ITEMS + class], an even number) belong to k_simulate_gpipe, which
// takes them two at a time and has no sweep at all (gpipe_finish); all other items belong to
// k_simulate.  Two kernels, so that the one without a sweep gets by with fewer registers.  Either
// launch numbers the pairs of its own items and a wavefront takes them with the stride of the grid
// (about one pair per wavefront for large lists: the hardware's dispatch order is the load
// balancing, so the order of the pairs is longest first, see PairOrder).

constexpr int64_t kSplitMinItems = 262144;     // default list length (candidates) from which two launches share the items

// The header is read through the constant address space: nothing writes it while a sweep runs,
// and a wave-uniform index then makes every read a scalar load that needs no vector register.
typedef const __attribute__((address_space(4))) int64_t* HdrPtr;
__device__ __forceinline__ Item decode_item_c(HdrPtr hdr, int64_t w) {
    int k = 0;
#pragma unroll
    for (int i = 1; i < kClasses; i++) k += (w >= hdr[H_ITEM_START + i]) ? 1 : 0;
    Item it;
    it.sh = 6 - k;
    it.pos0 = hdr[H_CLASS_START + k] + ((w - hdr[H_ITEM_START + k]) << k);
    it.class_end = hdr[H_CLASS_START + k + 1];
    return it;
}

// The order in which a launch takes its pairs is a table in the workspace (k_pair_order): entry q
// names the pair's first wave-item and says whether the next item belongs to the pair.  A pair
// never straddles two classes.
typedef const __attribute__((address_space(4))) int32_t* OrderPtr;

template <bool GPIPE_PAIRS>
__device__ __forceinline__ void simulate_all(const CostsDev& co, const ClusterDev& cl, const CandDev& ca,
                                             const Workspace& ws, const EventsDev& ev, const SimOut& out,
                                             Park& park) {
    const int lane = lane_id();
    const HdrPtr hdr = (HdrPtr)ws.hdr;
    // the wavefront's number as a scalar: the header words and the item ranges then come through
    // scalar loads, all requested at once, instead of a chain of dependent vector loads
    const int64_t wave0 = __builtin_amdgcn_readfirstlane((int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave));
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    int64_t W = hdr[H_NUM_ITEMS];                       // items that have room in the per-stage arrays
    if (W * kWave > ev.stage_cap) W = ev.stage_cap / kWave;
    const OrderPtr order = (OrderPtr)ws.order[GPIPE_PAIRS ? 1 : 0];
    const int64_t pairs = hdr[H_PAIRS + (GPIPE_PAIRS ? 1 : 0)];
    const int L = co.L;
    // Rounds of nwaves pairs, taken back and forth: a wavefront's pairs are w, 2n-1-w, 2n+w, ...  With
    // the pairs in order of falling length that gives every wavefront about the same total, so a
    // grid that is resident all at once ends together; with more wavefronts than pairs it is just
    // pair number = wavefront number and the hardware's dispatch order balances the load.
    for (int64_t r0 = 0; r0 < pairs; r0 += 2 * nwaves)
    for (int half = 0; half < 2; half++) {
        const int64_t q = half == 0 ? r0 + wave0 : r0 + 2 * nwaves - 1 - wave0;
        if (q >= pairs) continue;
        const int32_t e = order[q];
        const bool pair = e < 0;
        struct { int64_t w; } oa{e & 0x7fffffff}, ob{pair ? oa.w + 1 : oa.w};
        const Item ia = decode_item_c(hdr, oa.w);
        Item ib = ia;                                   // the same class: the next 64 >> sh candidates
        if (pair) ib.pos0 += (int64_t)1 << (6 - ia.sh);
        const int64_t posa = ia.pos0 + (lane >> ia.sh), posb = ib.pos0 + (lane >> ib.sh);
        Desc da{}, db{};
        if (posa < ia.class_end) da = ws.desc[posa];
        if (pair && posb < ib.class_end) db = ws.desc[posb];
        if (has_own_kernel(da)) da = Desc{};          // those candidates have a kernel of their own
        if (has_own_kernel(db)) db = Desc{};
        if constexpr (GPIPE_PAIRS) {
            // an even number of items per class and room for all of them (k_bins): always two, side by side
            const Desc two[2] = {da, db};
            simulate_items<2, false, true>(cl, ca, ws, ev, out, L, oa.w, ia.sh, two, lane, park);
        } else {
            const bool okA = oa.w < W, okB = pair && ob.w < W;
            // simulated together when every lane sees the same shape (pp, m, schedule) in both,
            // which neighbours in visiting order mostly do, else one after the other
            const bool same = okA && okB &&
                              __builtin_amdgcn_ballot_w64(((da.meta ^ db.meta) & 0xffff) != 0 || da.m != db.m) == 0;
            if (same) {
                const Desc two[2] = {da, db};
                simulate_items<2>(cl, ca, ws, ev, out, L, oa.w, ia.sh, two, lane, park);
            } else {
                if (okA) {
                    const Desc one[1] = {da};
                    simulate_items<1>(cl, ca, ws, ev, out, L, oa.w, ia.sh, one, lane, park);
                }
                if (okB) {
                    const Desc one[1] = {db};
                    simulate_items<1>(cl, ca, ws, ev, out, L, ob.w, ib.sh, one, lane, park);
                }
            }
        }
    }
}

__global__ __launch_bounds__(kSimBlock, 6) void k_simulate(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                           EventsDev ev, SimOut out) {
    // What only the epilogue needs is parked in LDS during the sweep (each lane its own slot),
    // so that the sweep runs in few enough registers for six wavefronts per SIMD.
    __shared__ Park park;
    simulate_all<false>(co, cl, ca, ws, ev, out, park);
}

// init_C > 0: the launch also does k_sim_init's work for the candidates [0, init_C) first (it runs beside
// k_simulate then, and one launch less stands in front of it on its stream).
__global__ __launch_bounds__(kSimBlock, 6) void k_simulate_gpipe(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                                 EventsDev ev, SimOut out, int64_t init_C) {
    __shared__ Park park;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < init_C; c += (int64_t)gridDim.x * blockDim.x)
        if (ev.status[c] != 0) out.batch_ns[c] = INT64_MAX;
    simulate_all<true>(co, cl, ca, ws, ev, out, park);
}

// Same contract as k_simulate for p2p_blocking = 2 (sends queue on their link): one item per
// wavefront turn, plain sweep.
__global__ __launch_bounds__(kSimBlock) void k_simulate_links(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                              EventsDev ev, SimOut out) {
    const int lane = lane_id();
    const int64_t wave0 = __builtin_amdgcn_readfirstlane((int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave));
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    int64_t W = ws.hdr[H_NUM_ITEMS];
    if (W * kWave > ev.stage_cap) W = ev.stage_cap / kWave;
    __shared__ Park park;
    for (int64_t w = wave0; w < W; w += nwaves) {
        const Item it = decode_item(ws.hdr, w);
        const int64_t pos = it.pos0 + (lane >> it.sh);
        Desc d{};
        if (pos < it.class_end) d = ws.desc[pos];
        if (has_own_kernel(d)) d = Desc{};
        const Desc one[1] = {d};
        simulate_items<1, true>(cl, ca, ws, ev, out, co.L, w, it.sh, one, lane, park);
    }
}

}  // namespace distsim
