// Timeline dump: start and end of every stage-task of selected candidates, i.e. the per-device
// event lists of Algorithm 1 reduced to their stage-tasks, plus the window of the gradient
// all-reduce events of every stage (Sec. 3.2: "when and which device will compute and
// communicate").
#pragma once
#include "kernels_build.hpp"

namespace distsim {

struct TimelineOut {
    const int64_t* sel;         // [n] candidate indices
    const int64_t* task_off;    // [n] first entry of the candidate's block in start / end
    int64_t* start;             // block layout [2][pp][m]: kind (0 forward, 1 backward), stage, micro-batch
    int64_t* end;
    int64_t* ar_start;          // [n][kMaxPP] start of the stage's first all-reduce event, -1 = none
    int64_t* ar_end;            // [n][kMaxPP] end of its last one
};

// One wavefront per selected candidate, lane = stage.  The sweep is written with explicit
// per-level predicates on x = level - s (see the level functions in kernels_simulate.hpp).
__global__ __launch_bounds__(64) void k_timeline(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                 const int32_t* __restrict__ status, int64_t n, TimelineOut out) {
    const int64_t q = blockIdx.x;
    if (q >= n) return;
    const int s = threadIdx.x;
    const int64_t c = out.sel[q];
    out.ar_start[q * kMaxPP + s] = -1;
    out.ar_end[q * kMaxPP + s] = -1;
    if (status[c] != 0) return;                      // uniform: the whole wavefront leaves
    const int L = co.L;
    const int pp = ca.pp[c], m = ca.m[c], dp = ca.dp[c], tp = ca.tp[c], sched = ca.schedule[c];
    const int64_t poff = ca.part_off[c];
    int v = 0;
    for (int i = co.V - 1; i >= 0; i--) if (co.variant_tp[i] == tp) v = i;
    const bool act = s < pp;
    int lo = 0, hi = 0;
    if (act) {
        if (poff >= 0) { lo = ca.part_pool[poff + s]; hi = ca.part_pool[poff + s + 1]; }
        else { lo = (int)(((int64_t)s * L) / pp); hi = (int)(((int64_t)(s + 1) * L) / pp); }
    }
    StageRow r;
    if (stage_row(cl, ws, L, kWave, s, pp, v, m, dp, tp, lo, hi, r) != 0) return;
    const int64_t pf_task = cl.blocking ? r.PF : 0, pb_task = cl.blocking ? r.PB : 0;
    const int64_t Fd = r.FC + r.FA + pf_task, Bd = r.BC + r.BA + pb_task;
    int64_t latF = __shfl_up(r.PF - pf_task, 1, kWave), latB = __shfl_down(r.PB - pb_task, 1, kWave);
    const bool hasL = act && s > 0, hasR = act && s + 1 < pp;

    int wq = pp - 1 - s; if (wq > m) wq = m;                 // 1F1B warm-up forwards
    const int offB = sched == 0 ? m + 2 * pp - 2 - 2 * s : 2 * pp - 1 - 2 * s;
    const int nlev = 2 * (m + pp - 1);
    int64_t* st = out.start + out.task_off[q];
    int64_t* en = out.end + out.task_off[q];
    int64_t own = 0;
    for (int lvl = 0; lvl < nlev; lvl++) {
        const int64_t fromL = __shfl_up(own, 1, kWave), fromR = __shfl_down(own, 1, kWave);
        const int x = lvl - s, y = x - offB;
        int jF = -1, jB = -1;
        if (act && x >= 0) {
            if (sched == 0) { if (x < m) jF = x; }
            else if (x <= wq) { if (x < m) jF = x; }
            else if ((x & 1) == 0 && x > 2 * wq && x < 2 * m) jF = x >> 1;
        }
        if (act && y >= 0) {
            if (sched == 0) { if (y < m) jB = y; }
            else if ((y & 1) == 0 && y < 2 * m) jB = y >> 1;
        }
        if (jF >= 0) {
            int64_t t0 = own;
            if (hasL && fromL + latF > t0) t0 = fromL + latF;
            own = t0 + Fd;
            st[((int64_t)0 * pp + s) * m + jF] = t0;
            en[((int64_t)0 * pp + s) * m + jF] = own;
        } else if (jB >= 0) {
            int64_t t0 = own;
            if (hasR && fromR + latB > t0) t0 = fromR + latB;
            own = t0 + Bd;
            st[((int64_t)1 * pp + s) * m + jB] = t0;
            en[((int64_t)1 * pp + s) * m + jB] = own;
        }
    }
    // data-parallel modelling: window of the gradient all-reduce events on this device
    if (!(act && dp > 1 && r.G > 0)) return;
    const int64_t endB = own;
    if (cl.bucket <= 0) {
        out.ar_start[q * kMaxPP + s] = endB;
        out.ar_end[q * kMaxPP + s] = endB + allreduce_ns(cl, dp, r.G);
        return;
    }
    const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
    const int64_t startB = endB - Bd;
    const int64_t tot_hi = ws.pbc[vr + hi] + ws.pba[rr + hi];
    const int64_t ar_cap = allreduce_ns(cl, dp, cl.bucket);
    int64_t acc = 0, t = 0, first = -1;
    for (int l = hi - 1; l >= lo; l--) {
        const int64_t ready = startB + (tot_hi - (ws.pbc[vr + l] + ws.pba[rr + l]));
        acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
        const int64_t k = (int64_t)udiv64((uint64_t)acc, (uint64_t)cl.bucket);
        if (k > 0) {
            const int64_t b0 = t > ready ? t : ready;
            if (first < 0) first = b0;
            t = b0 + k * ar_cap;
            acc -= k * cl.bucket;
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

}  // namespace distsim
