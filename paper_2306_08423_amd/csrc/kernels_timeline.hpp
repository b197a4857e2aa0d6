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

// Levels between two flushes of the staging ring = entries a stage can add to one row meanwhile.
#ifndef DISTSIM_TL_RING
#define DISTSIM_TL_RING 8
#endif
constexpr int kTlRing = DISTSIM_TL_RING;
constexpr int kTlRow = kTlRing + 1;      // padded: consecutive stages start in different LDS banks

// One wavefront per selected candidate, lane = stage.  The sweep is written with explicit
// per-level predicates on x = level - s (see the level functions in kernels_simulate.hpp).
// A stage's tasks of one kind come in micro-batch order, so the entries it produces between two
// flushes are one run of consecutive micro-batches of its row [kind][stage][.].  Start times are
// staged in an LDS ring per row; every kTlRing levels the wavefront writes the new runs out,
// kTlRing lanes per row and several rows per store, so that a store instruction touches a few cache lines
// instead of one per lane.  The end time is the start plus the row's task duration.
__global__ __launch_bounds__(64) void k_timeline(CostsDev co, ClusterDev cl, CandDev ca, Workspace ws,
                                                 const int32_t* __restrict__ status, int64_t n, TimelineOut out) {
    __shared__ int64_t ring[2][kMaxPP][kTlRow];
    __shared__ int64_t dur[2][kMaxPP];
    __shared__ int32_t done[2][kMaxPP], flushed[2][kMaxPP];
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
    const int64_t latF = dpp_i64<kDppWaveShr1>(r.PF - pf_task), latB = dpp_i64<kDppWaveShl1>(r.PB - pb_task);
    const bool hasL = act && s > 0, hasR = act && s + 1 < pp;
    dur[0][s] = Fd; dur[1][s] = Bd;
    flushed[0][s] = 0; flushed[1][s] = 0;

    int wq = pp - 1 - s; if (wq > m) wq = m;                 // 1F1B warm-up forwards
    const int offB = sched == 0 ? m + 2 * pp - 2 - 2 * s : 2 * pp - 1 - 2 * s;
    const int nlev = 2 * (m + pp - 1);
    int64_t* st = out.start + out.task_off[q];
    int64_t* en = out.end + out.task_off[q];
    const int sub = s / kTlRing, e = s & (kTlRing - 1);           // flush role: row within a group of 4, entry
    int64_t own = 0;
    int nF = 0, nB = 0;                                      // tasks of each kind done so far
    for (int lvl = 0; lvl < nlev; lvl++) {
        const int64_t fromL = dpp_i64<kDppWaveShr1>(own), fromR = dpp_i64<kDppWaveShl1>(own);
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
            ring[0][s][jF & (kTlRing - 1)] = t0;
            nF = jF + 1;
        } else if (jB >= 0) {
            int64_t t0 = own;
            if (hasR && fromR + latB > t0) t0 = fromR + latB;
            own = t0 + Bd;
            ring[1][s][jB & (kTlRing - 1)] = t0;
            nB = jB + 1;
        }
        if ((lvl & (kTlRing - 1)) != kTlRing - 1 && lvl != nlev - 1) continue;
        // flush: rows [kind][stage], the run [flushed, done) of each
        done[0][s] = nF; done[1][s] = nB;
        __syncthreads();
        for (int kind = 0; kind < 2; kind++) {
            if (__builtin_amdgcn_ballot_w64(done[kind][s] > flushed[kind][s]) == 0) continue;
            for (int r0 = 0; r0 < pp; r0 += kWave / kTlRing) {
                const int row = r0 + sub;
                if (row < pp) {
                    const int j = flushed[kind][row] + e;
                    if (j < done[kind][row]) {
                        const int64_t t0 = ring[kind][row][j & (kTlRing - 1)];
                        const int64_t i = ((int64_t)kind * pp + row) * m + j;
                        st[i] = t0;
                        en[i] = t0 + dur[kind][row];
                    }
                }
            }
        }
        __syncthreads();
        flushed[0][s] = nF; flushed[1][s] = nB;
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
