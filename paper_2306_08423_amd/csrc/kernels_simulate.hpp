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

__global__ __launch_bounds__(256, 8) void k_simulate(CostsDev co, ClusterDev cl, CandDev ca,
                                                                    Workspace ws, EventsDev ev, SimOut out) {
    const int lane = lane_id();
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    int64_t W = ws.hdr[H_NUM_ITEMS];
    if (W * kWave > ev.stage_cap) W = ev.stage_cap / kWave;
    const int L = co.L;
    const double ninf = -__builtin_huge_val();
    // What only the epilogue needs is parked in LDS during the sweep (each lane its own slot),
    // so that the sweep runs in few enough registers for eight wavefronts per SIMD.
    __shared__ int64_t park_comp[256], park_comm[256], park_ar[256];
    __shared__ int32_t park_cand[256], park_dp[256], park_misc[256];
    const int slot = threadIdx.x;

    for (int64_t w = wave0; w < W; w += nwaves) {
        const Item it = decode_item(ws.hdr, w);
        const int width = 1 << it.sh;
        const int s = lane & (width - 1);
        const int64_t pos = it.pos0 + (lane >> it.sh);
        Desc d{};
        if (pos < it.class_end) d = ws.desc[pos];
        int pp = d.meta & 0xff;
        const int sched = (d.meta >> 8) & 0xff, v = d.meta >> 16, dp = d.meta ? d.dp : 1;
        const int64_t c = d.cand;
        // the stage's composed events, regenerated from the layer-event tables
        int lo = 0, hi = 0;
        if (s < pp) {
            if (d.poff >= 0) { lo = ca.part_pool[d.poff + s]; hi = ca.part_pool[d.poff + s + 1]; }
            else { lo = (int)(((int64_t)s * L) / pp); hi = (int)(((int64_t)(s + 1) * L) / pp); }
        }
        StageRow r;
        const int drop = stage_row(cl, ws, L, width, s, pp, v, d.m, dp, (int)d.spare, lo, hi, r);
        if (drop) {
            if (s == 0 && pp > 0) { ev.status[c] = drop; ev.num_events[c] = 0; out.batch_ns[c] = INT64_MAX; }
            pp = 0;
        }
        const bool act = s < pp;
        const int m = act ? d.m : 0;
        const int64_t i = w * kWave + lane;
        double Fd, Bd, pfL, pbR;
        int64_t comp1, comm1, AR;            // per-micro-batch computation / communication, trailing all-reduce
        bool has_ar;                         // the stage has gradient bytes to reduce over dp > 1 ranks
        {
            AR = cl.bucket > 0 ? 0 : allreduce_ns(cl, dp, r.G);
            has_ar = act && dp > 1 && r.G > 0;
            comp1 = r.FC + r.BC; comm1 = r.FA + r.BA + r.PF + r.PB;
            // p2p on the incoming edges (the neighbours' outgoing events): latency of the edge, or,
            // when the sender is occupied by it, part of the sender's task; -inf = no edge
            const int64_t pf_task = cl.blocking ? r.PF : 0, pb_task = cl.blocking ? r.PB : 0;
            Fd = (double)(r.FC + r.FA + pf_task); Bd = (double)(r.BC + r.BA + pb_task);
            pfL = from_prev_lane((double)(r.PF - pf_task)); pbR = from_next_lane((double)(r.PB - pb_task));
        }
        if (!(act && s > 0)) pfL = ninf;
        if (!(act && s + 1 < pp)) pbR = ninf;
        park_comp[slot] = comp1; park_comm[slot] = comm1; park_ar[slot] = AR;
        park_cand[slot] = (int32_t)c; park_dp[slot] = dp;
        park_misc[slot] = lo | (hi << 8) | ((int)has_ar << 16) | (v << 17);

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

        // 1F1B past its warm-up runs forwards on even x and backwards on odd x.  When every
        // candidate of the wavefront is 1F1B with one pp, a level that has both kinds therefore
        // splits the lanes by parity, and one merged operand (previous lane for the forward
        // lanes, next lane for the backward lanes) feeds a single task step.
        const int ppu = __builtin_amdgcn_readfirstlane(wave_max_i32(pp));
        const bool par_ok = width >= 2 && __builtin_amdgcn_ballot_w64(act && (sched == 0 || pp != ppu)) == 0;
        const bool even_s = (s & 1) == 0;
        const double latE = even_s ? pfL : pbR, durE = even_s ? Fd : Bd;     // roles on even levels
        const double latO = even_s ? pbR : pfL, durO = even_s ? Bd : Fd;     // roles on odd levels
        const int adrE = (even_s ? lane - 1 : lane + 1) * 4;

        double own = 0.0;
        for (int l0 = 0; l0 < nlev; l0 += 32) {
            const int x0 = l0 - s;
            const uint32_t even_x = (x0 & 1) ? 0x55555555u : 0xaaaaaaaau;       // levels with even x
            uint32_t PFb = level_bits(-x0, f1hi - x0) | (level_bits(f2lo - x0, f2hi - x0) & even_x);
            uint32_t PBb = level_bits(blo - x0, bhi - x0);
            if (sched != 0) PBb &= ((blo - x0) & 1) ? 0x55555555u : 0xaaaaaaaau;   // x - blo even
            if (!act) { PFb = 0; PBb = 0; }
            // chunk-relative level ranges in which any lane has a forward / a backward task
            const uint32_t orF = wave_or_u32(PFb), orB = wave_or_u32(PBb);
            if ((orF | orB) == 0) continue;
            const int firstF = orF ? __builtin_clz(orF) : 64, lastF = orF ? 31 - __builtin_ctz(orF) : -1;
            const int firstB = orB ? __builtin_clz(orB) : 64, lastB = orB ? 31 - __builtin_ctz(orB) : -1;
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
                if (inF && inB) {
                    if (par_ok) {
                        uint32_t Pc = PFb | PBb;
                        int j = 0;
                        if (((l0 + k) & 1) && j < len) {
                            double nb = from_pair_partner(own);
                            DISTSIM_STEP_ONE(Pc, nb, latO, durO);
                            j++;
                        }
                        for (; j + 1 < len; j += 2) {
                            double nb = from_lanes(own, adrE);
                            DISTSIM_STEP_ONE(Pc, nb, latE, durE);
                            double nb2 = from_pair_partner(own);
                            DISTSIM_STEP_ONE(Pc, nb2, latO, durO);
                        }
                        if (j < len) {
                            double nb = from_lanes(own, adrE);
                            DISTSIM_STEP_ONE(Pc, nb, latE, durE);
                        }
                        PFb = shl32(PFb, len); PBb = shl32(PBb, len);
                    } else {
                        for (int j = 0; j < len; j++) {
                            double fromL = from_prev_lane(own);
                            double fromR = from_next_lane(own);
                            DISTSIM_STEP_BOTH();
                        }
                    }
                } else if (inF) {
                    for (int j = 0; j < len; j++) {
                        double fromL = from_prev_lane(own);
                        DISTSIM_STEP_ONE(PFb, fromL, pfL, Fd);
                    }
                    PBb = shl32(PBb, len);
                } else if (inB) {
                    for (int j = 0; j < len; j++) {
                        double fromR = from_next_lane(own);
                        DISTSIM_STEP_ONE(PBb, fromR, pbR, Bd);
                    }
                    PFb = shl32(PFb, len);
                } else {
                    PFb = shl32(PFb, len); PBb = shl32(PBb, len);
                }
                k = e;
            }
            (void)kmask; (void)kmask2;
        }

        // data-parallel modelling: gradient all-reduce after (or overlapped with) the last backward
        const int64_t endB = (int64_t)own;
        const int64_t AR_ = park_ar[slot];
        const int misc = park_misc[slot];
        const bool has_ar_ = (misc >> 16) & 1;
        int64_t finish = endB + AR_, ar_busy = AR_, nar = has_ar_ ? 1 : 0;
        if (has_ar_ && cl.bucket > 0) {
            const int lo = misc & 0xff, hi = (misc >> 8) & 0xff, v = misc >> 17, dp = park_dp[slot];
            const size_t vr = (size_t)v * (L + 1), rr = (size_t)(v * kMaxPP + pp - 1) * (L + 1);
            const int64_t startB = endB - (int64_t)Bd;
            const int64_t tot_hi = ws.pbc[vr + hi] + ws.pba[rr + hi];
            const int64_t ar_cap = allreduce_ns(cl, dp, cl.bucket);
            int64_t acc = 0, t = 0;
            ar_busy = 0; nar = 0;
            for (int l = hi - 1; l >= lo; l--) {
                const int64_t ready = startB + (tot_hi - (ws.pbc[vr + l] + ws.pba[rr + l]));
                acc += ws.pg[vr + l + 1] - ws.pg[vr + l];
                const int64_t k = (int64_t)udiv64((uint64_t)acc, (uint64_t)cl.bucket);
                if (k > 0) {
                    t = (t > ready ? t : ready) + k * ar_cap;
                    ar_busy += k * ar_cap;
                    nar += k;
                    acc -= k * cl.bucket;
                }
                if (l == lo && acc > 0) {
                    const int64_t dlast = allreduce_ns(cl, dp, acc);
                    t = (t > ready ? t : ready) + dlast;
                    ar_busy += dlast;
                    nar += 1;
                }
            }
            finish = t > endB ? t : endB;
        }
        nar = group_sum(nar, width);
        const int64_t batch = group_max(act ? finish : 0, width);
        // lanes outside a candidate have m = 0 and zero rows: they store zeros
        const int64_t comp = (int64_t)m * park_comp[slot];
        const int64_t comm = act ? (int64_t)m * park_comm[slot] + ar_busy : 0;
        out.comp_busy[i] = comp;
        out.comm_busy[i] = comm;
        if (out.util) out.util[i] = batch > 0 ? (double)comp / (double)batch : 0.0;
        if (act && s == 0) {
            const int64_t cc = park_cand[slot];
            out.batch_ns[cc] = batch;
            ev.num_events[cc] = 2ll * m * pp + 2ll * m * (pp - 1) + nar;
        }
    }
}

}  // namespace distsim
