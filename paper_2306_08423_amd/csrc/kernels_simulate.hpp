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
// chosen such that every dependency of a level-l task lies in a lower level:
//   GPipe  F(s,j): s + j                         B(s,j): (m + pp - 1) + (pp - 1 - s) + j
//   1F1B   F(s,j): s + j        (j <= w_s)       B(s,j): 2 pp - 1 - s + 2 j
//                  s + 2 j      (j >  w_s)       w_s = min(pp - 1 - s, m) warm-up forwards
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

// bits of the chunk-relative levels a..b (inclusive), bit 31 = level 0
__device__ __forceinline__ uint32_t level_bits(int a, int b) {
    const bool any = a <= b && a <= 31 && b >= 0;
    const int lo = a < 0 ? 0 : (a > 31 ? 31 : a);
    const int hi = b > 31 ? 31 : (b < 0 ? 0 : b);
    const uint32_t r = (0xffffffffu >> lo) & (0xffffffffu << (31 - hi));
    return any ? r : 0u;
}

// One level for the lanes whose pattern bit is set: own = max(own, nb + lat) + dur.
// Requires EXEC == all ones on entry (wave-uniform control flow, full wavefronts) and leaves
// it so.  The trailing s_nop keeps two wait states between the write of `own` and the DPP
// read that follows.
#define DISTSIM_STEP_ONE(bits, nb, lat, dur)                                   \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[p], %[k], %[p], %[p]\n\t"                        \
        "s_mov_b64 exec, %[k]\n\t"                                            \
        "v_add_f64 %[t], %[t], %[c]\n\t"                                      \
        "v_max_f64 %[t], %[t], %[o]\n\t"                                      \
        "v_add_f64 %[o], %[t], %[d]\n\t"                                      \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o] "+v"(own), [t] "+v"(nb), [p] "+v"(bits), [k] "=&s"(kmask)       \
        : [c] "v"(lat), [d] "v"(dur))

#define DISTSIM_STEP_BOTH()                                                    \
    asm volatile(                                                              \
        "v_add_co_u32_e64 %[pf], %[kf], %[pf], %[pf]\n\t"                    \
        "v_add_co_u32_e64 %[pb], %[kb], %[pb], %[pb]\n\t"                    \
        "s_mov_b64 exec, %[kf]\n\t"                                           \
        "v_add_f64 %[tl], %[tl], %[cl]\n\t"                                   \
        "v_max_f64 %[tl], %[tl], %[o]\n\t"                                    \
        "v_add_f64 %[o], %[tl], %[df]\n\t"                                    \
        "s_mov_b64 exec, %[kb]\n\t"                                           \
        "v_add_f64 %[tr], %[tr], %[cr]\n\t"                                   \
        "v_max_f64 %[tr], %[tr], %[o]\n\t"                                    \
        "v_add_f64 %[o], %[tr], %[db]\n\t"                                    \
        "s_mov_b64 exec, -1\n\t"                                              \
        "s_nop 0"                                                              \
        : [o] "+v"(own), [tl] "+v"(fromL), [tr] "+v"(fromR), [pf] "+v"(PFb), [pb] "+v"(PBb),  \
          [kf] "=&s"(kmask), [kb] "=&s"(kmask2)                               \
        : [cl] "v"(pfL), [cr] "v"(pbR), [df] "v"(Fd), [db] "v"(Bd))

__global__ __launch_bounds__(256) void k_simulate(CostsDev co, ClusterDev cl, Workspace ws, EventsDev ev,
                                                  SimOut out) {
    const int lane = lane_id();
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    int64_t W = ws.hdr[H_NUM_ITEMS];
    if (W * kWave > ev.stage_cap) W = ev.stage_cap / kWave;
    const int64_t cap = ev.stage_cap;
    const int L = co.L;
    const double ninf = -__builtin_huge_val();

    for (int64_t w = wave0; w < W; w += nwaves) {
        const Item it = decode_item(ws.hdr, w);
        const int width = 1 << it.sh;
        const int s = lane & (width - 1);
        const int64_t pos = it.pos0 + (lane >> it.sh);
        int4 dd = make_int4(0, 0, 0, 0);                   // cand, meta, m, dp
        if (pos < it.class_end) dd = *reinterpret_cast<const int4*>(&ws.desc[pos]);
        const int pp = dd.y & 0xff, sched = (dd.y >> 8) & 0xff, v = dd.y >> 16, dp = dd.y ? dd.w : 1;
        const int64_t c = dd.x;
        const bool act = s < pp;
        const int m = act ? dd.z : 0;
        const int64_t i = w * kWave + lane;
        // rows of lanes outside a candidate are zero-filled by event generation
        const int64_t FC = ev.stage_tab[0 * cap + i], FA = ev.stage_tab[1 * cap + i];
        const int64_t BC = ev.stage_tab[2 * cap + i], BA = ev.stage_tab[3 * cap + i];
        const int64_t PF = ev.stage_tab[4 * cap + i], PB = ev.stage_tab[5 * cap + i];
        const int64_t AR = ev.stage_tab[7 * cap + i];
        // p2p latency on the incoming edges (the neighbours' outgoing events); -inf = no edge
        double pfL = from_prev_lane((double)PF), pbR = from_next_lane((double)PB);
        if (!(act && s > 0)) pfL = ninf;
        if (!(act && s + 1 < pp)) pbR = ninf;
        const double Fd = (double)(FC + FA), Bd = (double)(BC + BA);

        // level windows of this lane, expressed on x = level - s:
        //   forward  x in [0, f1hi]  and  even x in [f2lo, f2hi]
        //   backward x in [blo, bhi], every x (GPipe) or every second x (1F1B)
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
        const int nlev = __builtin_amdgcn_readfirstlane(wave_max_i32(act ? 2 * (m + pp - 1) : 0));

        double own = 0.0;
        for (int l0 = 0; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;       // levels with even x
            uint32_t PFb = level_bits(-x0, f1hi - x0) | (level_bits(f2lo - x0, f2hi - x0) & even_x);
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            if (sched != 0) PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;   // x - blo even
            if (!act) { PFb = 0; PBb = 0; }
            const bool anyF = __builtin_amdgcn_ballot_w64(PFb != 0) != 0;
            const bool anyB = __builtin_amdgcn_ballot_w64(PBb != 0) != 0;
            const int n = nlev - l0 < 32 ? nlev - l0 : 32;
            uint64_t kmask, kmask2;
            if (anyF && anyB) {
                for (int k = 0; k < n; k++) {
                    double fromL = from_prev_lane(own);
                    double fromR = from_next_lane(own);
                    DISTSIM_STEP_BOTH();
                }
            } else if (anyF) {
                for (int k = 0; k < n; k++) {
                    double fromL = from_prev_lane(own);
                    DISTSIM_STEP_ONE(PFb, fromL, pfL, Fd);
                }
            } else if (anyB) {
                for (int k = 0; k < n; k++) {
                    double fromR = from_next_lane(own);
                    DISTSIM_STEP_ONE(PBb, fromR, pbR, Bd);
                }
            }
            (void)kmask; (void)kmask2;
        }

        // data-parallel modelling: gradient all-reduce after (or overlapped with) the last backward
        const int64_t endB = (int64_t)own;
        int64_t finish = endB + AR, ar_busy = AR;
        if (act && cl.bucket > 0) {
            finish = endB; ar_busy = 0;
            if (dp > 1) {
                const int lay = ev.stage_layers[i];
                const int lo = lay & 0xff, hi = lay >> 8;
                const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
                const int64_t startB = endB - (BC + BA);
                const int64_t tot_hi = ws.pbc[vr + hi] + ws.pba[rr + hi];
                const int64_t ar_cap = allreduce_ns(cl, dp, cl.bucket);
                int64_t acc = 0, t = 0;
                for (int l = hi - 1; l >= lo; l--) {
                    const int64_t ready = startB + (tot_hi - (ws.pbc[vr + l] + ws.pba[rr + l]));
                    acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
                    const int64_t k = (int64_t)udiv64((uint64_t)acc, (uint64_t)cl.bucket);
                    if (k > 0) {
                        t = (t > ready ? t : ready) + k * ar_cap;
                        ar_busy += k * ar_cap;
                        acc -= k * cl.bucket;
                    }
                    if (l == lo && acc > 0) {
                        const int64_t d = allreduce_ns(cl, dp, acc);
                        t = (t > ready ? t : ready) + d;
                        ar_busy += d;
                    }
                }
                finish = t > endB ? t : endB;
            }
        }
        const int64_t batch = group_max(act ? finish : 0, width);
        // lanes outside a candidate have m = 0 and zero rows: they store zeros
        const int64_t comp = (int64_t)m * (FC + BC);
        const int64_t comm = act ? (int64_t)m * (FA + BA + PF + PB) + ar_busy : 0;
        out.comp_busy[i] = comp;
        out.comm_busy[i] = comm;
        if (out.util) out.util[i] = batch > 0 ? (double)comp / (double)batch : 0.0;
        if (act && s == 0) out.batch_ns[c] = batch;
    }
}

}  // namespace distsim
