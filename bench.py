#!/usr/bin/env python3
"""Throughput of the batched strategy evaluation on one MI355X.

One step = one pass of the whole hot path over one resident batch of candidates:
distsim_build_events -> distsim_simulate -> distsim_search.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# fp64 add / max issue rate of the vector ALUs: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.
# (The published 78.6 TFLOP/s counts an FMA as two; add and max are one flop each.)
ALU_PEAK_TFLOPS = 256 * 4 * 16 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0
FLOPS_PER_TASK = 3          # cross-stage end + p2p, max with the device's previous end, + duration


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2306_08423_amd", "csrc")
    for f in sorted(os.listdir(d)):
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload: str):
    """HBM bytes per step of the two simulate kernels (k_simulate, k_simulate_gpipe) from the
    committed counter summary; None when the kernel sources changed after the counters were taken."""
    p = os.path.join(ROOT, "profiles", f"pmc_k_simulate_{workload}.txt")
    if not os.path.exists(p):
        return None
    vals = {}
    for line in open(p):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    if vals.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    try:
        return float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def variant_workloads(w, n):
    """A seeded sample of n candidates of the workload, once per reading of the p2p events and per
    further schedule: (name, workload, kernel that does the variant's work, mask of the candidates
    that kernel simulates)."""
    import numpy as np
    from workloads import Workload, subset
    from workloads.schedules import chain, dapple_lists, gpipe_lists, pack_schedule, pack_schedules

    idx = np.sort(np.random.default_rng(11).choice(len(w.cand["pp"]), n, replace=False))
    base = subset(w, idx)
    L = int(w.costs["L"])
    everyone = np.ones(n, bool)

    def copy_cand():
        return {k: v.copy() for k, v in base.cand.items()}

    yield "default", base, "k_simulate", everyone
    for name, blocking in (("p2p_blocking_1", 1), ("serialised_links", 2)):
        cl = dict(base.cluster)
        cl["p2p_blocking"] = blocking
        yield name, Workload(base.name, base.costs, cl, base.cand), "k_simulate", everyone
    cand = copy_cand()
    cand["schedule"] = np.where(cand["schedule"] == 1, 2, cand["schedule"]).astype(np.uint8)
    yield "asynchronous", Workload(base.name, base.costs, dict(base.cluster), cand), "k_simulate", cand["schedule"] == 2
    # interleaved: two chunks per device, uniform partition, m rounded up to a multiple of pp
    cand = copy_cand()
    pp, m = base.cand["pp"].astype(np.int64), base.cand["m"].astype(np.int64)
    take = (pp >= 2) & (2 * pp <= min(L, 64))
    cand["m"] = np.where(take, ((m + pp - 1) // pp) * pp, m).astype(np.int32)
    cand["schedule"] = np.where(take, 3, cand["schedule"]).astype(np.uint8)
    cand["part_off"] = np.where(take, -1, cand["part_off"]).astype(np.int64)
    cand["chunks"] = np.where(take, 2, 1).astype(np.int32)
    yield "interleaved_2_chunks", Workload(base.name, base.costs, dict(base.cluster), cand), "k_simulate_virtual", take
    # explicit lists: the two built-in orders written out, for a few (pp, m) shapes
    cand = copy_cand()
    shapes = {4: 16, 8: 32, 16: 64}
    blocks, ids = [], np.zeros((65, 2), np.int32)
    for p_, m_ in shapes.items():
        for sc in (0, 1):
            ids[p_, sc] = len(blocks)
            blocks.append(pack_schedule(p_, chain(p_), m_, p_, 1, gpipe_lists(p_, m_) if sc == 0 else dapple_lists(p_, m_)))
    take = np.isin(pp, list(shapes)) & (base.cand["schedule"] <= 1)
    m_of = np.zeros(65, np.int64)
    for p_, m_ in shapes.items():
        m_of[p_] = m_
    cand["m"] = np.where(take, m_of[pp], m).astype(np.int32)
    cand["chunks"] = np.where(take, ids[pp, np.minimum(base.cand["schedule"], 1)], 0).astype(np.int32)
    cand["schedule"] = np.where(take, 4, cand["schedule"]).astype(np.uint8)
    cand["schedule_off"], cand["schedule_words"] = pack_schedules(blocks)
    yield "explicit_lists", Workload(base.name, base.costs, dict(base.cluster), cand), "k_simulate_explicit", take


def time_variants(ds, ctx, w, n):
    """The three calls on every workload of variant_workloads: ms per step and the time of the
    kernel that does the variant's work (HIP events of the library)."""
    import torch

    res = {"sample": f"{n} seeded candidates of {w.name}"}
    for name, wv, kernel, counted in variant_workloads(w, n):
        dwv = ds.upload(wv, ctx.device)
        evv = ds.alloc_events(ctx, dwv.L, dwv.V, dwv.C, ds.stage_entries(wv.cand["pp"]), table=False)
        outv = ds.alloc_outputs(ctx, evv, util=True)
        bestv, scr = ds.alloc_search(ctx, dwv.C)

        def stepv():
            ds.distsim_build_events(ctx, dwv, evv)
            ds.distsim_simulate(ctx, dwv, evv, outv)
            ds.distsim_search(ctx, outv.batch_ns, dwv.C, bestv, scr)
        stepv()
        torch.cuda.synchronize()
        ctx.timing_enable(True)
        t0 = time.perf_counter()
        for _ in range(5):
            stepv()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        ktv = ctx.timing_read()
        ctx.timing_enable(False)
        ms, cnt = ktv[kernel]
        ok = (evv.status[:dwv.C] == 0).cpu().numpy()
        n_counted = int((ok & counted).sum())
        k_ms = ms / max(cnt, 1)
        res[name] = {"candidates": int(dwv.C), "valid": int(ok.sum()), "ms_per_step": dt * 1e3, "kernel": kernel,
                     "kernel_ms": k_ms, "kernel_candidates": n_counted,
                     "kernel_candidates_per_s": n_counted / (k_ms / 1e3) if k_ms > 0 else None}
        if name == "explicit_lists":
            # the schedules are turned into programs once per distsim_build_events (k_simulate_explicit's
            # timer spans the kernel that runs the candidates from them and the one for schedules without)
            cms, ccnt = ktv["k_compile_schedules"]
            res[name]["compile_schedules_ms"] = cms / max(ccnt, 1)
            res[name]["schedules"] = int(len(wv.cand["schedule_off"]) - 1)
        del dwv, evv, outv, bestv, scr
    return res


def replicated_events(w, num_events, status) -> int:
    """Events of the full timeline that Algorithm 1 and the data-parallel modelling step build: the pp
    distinct device lists are appended to all tp devices of a stage and duplicated dp times."""
    import numpy as np
    ok = status == 0
    rep = w.cand["tp"].astype(np.int64) * w.cand["dp"].astype(np.int64)
    return int((num_events[ok] * rep[ok]).sum())


def measure(ds, torch, ctx, w, steps, warmup, table=False):
    """One workload through the three calls: `steps` timed steps with the library's per-kernel timers
    off (the headline), then the same number with them on (per-kernel times, span of the two sweep
    kernels).  Returns the figures and the device buffers (for the later sections)."""
    import numpy as np
    from workloads import total_stages
    dw = ds.upload(w, ctx.device)
    ev = ds.alloc_events(ctx, dw.L, dw.V, dw.C, ds.stage_entries(w.cand["pp"]), table=table)
    out = ds.alloc_outputs(ctx, ev, util=True)
    best, scratch = ds.alloc_search(ctx, dw.C)

    def step():
        ds.distsim_build_events(ctx, dw, ev)
        ds.distsim_simulate(ctx, dw, ev, out)
        ds.distsim_search(ctx, out.batch_ns, dw.C, best, scratch)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # second pass, same launches: HIP events of the library around every kernel, on the stream it runs on
    ctx.timing_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    kt = ctx.timing_read()
    ctx.timing_enable(False)
    C, S = dw.C, total_stages(w)
    m, pp = w.cand["m"].astype(np.int64), w.cand["pp"].astype(np.int64)
    tasks = int((2 * m * pp).sum())
    # stage-tasks that the level sweep visits one by one: GPipe candidates are not among them (their end
    # times come from the closed form of the same recurrence) unless sends queue on their links
    links = int(w.cluster.get("p2p_blocking", 0)) == 2
    visited = np.ones(C, bool) if links else w.cand["schedule"] != 0
    swept_tasks = int((2 * m * pp)[visited].sum())
    if not links:
        # nor are the warm-up forwards of the early-backward schedules (closed form too): stage s runs
        # min(pp - s, m) of them; summed over the stages that is pp (pp + 1) / 2 less the part beyond m
        k = np.maximum(pp - m, 0)
        warm = pp * (pp + 1) // 2 - k * (k + 1) // 2
        swept_tasks -= int(warm[visited].sum())
    status = ev.status[:C].cpu().numpy()
    num_events = ev.num_events[:C].cpu().numpy()
    sim_ms, sim_n = kt["k_simulate"]
    gp_ms, gp_n = kt["k_simulate_gpipe"]
    sim_avg_s = sim_ms / max(sim_n, 1) / 1e3
    # algorithmic HBM bytes of the sweep per launch: descriptor in (32 B), batch_ns and num_events out
    # (16 B) per candidate; partition byte in (1 B) and comp / comm / util out (24 B) per stage
    sim_bytes = C * (32 + 16) + S * (1 + 24)
    res = {
        "C": C, "S": S, "tasks": tasks, "swept_tasks": swept_tasks, "dt": dt, "kt": kt, "valid": int((status == 0).sum()),
        "events": int(num_events.sum()), "events_replicated": replicated_events(w, num_events, status),
        "sim_avg_s": sim_avg_s, "sim_launches": sim_n, "gpipe_ms": gp_ms / max(gp_n, 1), "sim_bytes": sim_bytes,
    }
    return res, (dw, ev, out, best, scratch, step)


def read_valu_instructions(workload: str):
    """VALU wave-instructions per step of the two simulate kernels from the committed counter summary
    (profiles/pmc_sq_bench_<workload>.txt); None when there is none or the kernel sources changed since."""
    p = os.path.join(ROOT, "profiles", f"pmc_sq_bench_{workload}.txt")
    if not os.path.exists(p):
        return None
    kernel, total, ok = None, 0.0, False
    for line in open(p):
        if line.startswith("# kernel_source_sha256_16:"):
            ok = line.split(":", 1)[1].strip() == kernel_source_hash()
        elif line.startswith("#"):
            continue
        elif not line.startswith(" "):
            kernel = line.strip()
        elif kernel in ("k_simulate", "k_simulate_gpipe"):
            f = line.split()
            if len(f) == 2 and f[0] == "SQ_INSTS_VALU":
                total += float(f[1])
    return total if ok and total > 0 else None


def sweep_rooflines(r, traffic, copy_gbs, valu=None):
    """The two views of the sweep kernels (k_simulate and k_simulate_gpipe side by side)."""
    hbm = {
        "kernel": "k_simulate || k_simulate_gpipe", "bound": "hbm",
        "achieved": r["sim_bytes"] / r["sim_avg_s"] / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "traffic": traffic, "algorithmic_bytes_per_launch": r["sim_bytes"],
        "avg_launch_ms": r["sim_avg_s"] * 1e3, "launches": r["sim_launches"],
        "launch_ms": {"span": r["sim_avg_s"] * 1e3, "k_simulate_gpipe": r["gpipe_ms"]},
        "note": "span of the two sweep kernels from HIP events on the caller's stream around fork and join, "
                "taken in a second pass of the same steps with the library's timers on; the sweep is bound by "
                "VALU issue, not by HBM (see roofline_alu)",
    }
    hbm["frac"] = hbm["achieved"] / HBM_PEAK_GBS
    if copy_gbs:
        hbm["frac_of_measured_copy"] = hbm["achieved"] / copy_gbs
    alu = {
        "kernel": "k_simulate || k_simulate_gpipe", "bound": "alu",
        "achieved": FLOPS_PER_TASK * r["swept_tasks"] / r["sim_avg_s"] / 1e12, "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
        "swept_stage_tasks": r["swept_tasks"],
        "derivation": "3 fp64 operations per stage-task that the level sweep visits (producer end + p2p, max with "
                      "the device's previous end, + duration; the stage-tasks of GPipe candidates and the warm-up "
                      "forwards of the other schedules, whose end times come from a closed form, are not counted) against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz "
                      "= 39.3 T non-FMA fp64 operations/s (the published 78.6 TFLOP/s counts an FMA as two)",
    }
    alu["frac"] = alu["achieved"] / alu["peak"]
    alu["frac_of_published_fp64_peak"] = alu["achieved"] / 78.6
    if valu:
        # how full the vector issue slots are, whatever the instructions do: counted wave-instructions of
        # both kernels x 4 cycles each against 1024 SIMDs x 2.4 GHz over the span
        alu["valu_instructions_per_launch"] = valu
        alu["valu_issue_frac"] = valu * 4 / (1024 * 2.4e9 * r["sim_avg_s"])
    return hbm, alu


def copy_bandwidth(torch, device, nbytes=1 << 30, reps=10):
    """Device-to-device copy of nbytes, timed with HIP events: read + write bytes per second in GB/s."""
    src = torch.empty(nbytes, dtype=torch.uint8, device=device)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    return 2 * nbytes / (ms / 1e3) / 1e9


def fill_bandwidth(torch, device, nbytes=1 << 30, reps=10):
    """A plain fill of nbytes of device memory, timed with HIP events: written bytes per second in
    GB/s, the rate this machine reaches for a kernel that only writes (the timeline dump is one)."""
    dst = torch.empty(nbytes // 8, dtype=torch.int64, device=device)
    dst.fill_(1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.fill_(1)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del dst
    return nbytes / (ms / 1e3) / 1e9


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="hetero64", help="hetero64 (default), gpt96, gpt48, gpt24")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-table", dest="no_stage_table", action="store_false",
                    help="also write the optional per-stage event table during event generation")
    ap.add_argument("--timeline", type=int, default=20000,
                    help="also dump the stage-task timelines of this many seeded candidates (0 = skip)")
    ap.add_argument("--ingest", type=int, default=4_000_000,
                    help="also time the steps in front of event generation (operator dedup, communication "
                         "event times) on this many seeded records (0 = skip)")
    ap.add_argument("--variants", type=int, default=100_000,
                    help="also time the other readings and schedules (blocking p2p, serialised links, asynchronous, "
                         "interleaved, explicit lists) on this many seeded candidates of the workload (0 = skip)")
    ap.add_argument("--search", type=int, default=1 << 27,
                    help="also time the argmin alone over this many seeded batch times, a list long enough for "
                         "HBM to bound it (0 = skip)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-copy", action="store_true",
                    help="skip the timed 1 GiB device-to-device copy and 1 GiB fill (the HBM bandwidth this box reaches "
                         "for read + write and for writes alone; the copy's known traffic also scales the HBM "
                         "counters of a profiler run)")
    ap.add_argument("--second", default="gpt96",
                    help="also time the three calls on this workload, the one with the most work per candidate "
                         "(none = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library evaluates candidates on ONE GPU; --gpus must be 1 "
              "(candidates would be sharded across GPUs with a 16-byte MINLOC exchange, which is not built)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2306_08423_amd as ds
    from workloads import make_workload, subset

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    w = make_workload(args.workload)
    ctx = ds.Context(0)
    res, (dw, ev, out, best, scratch, step) = measure(ds, torch, ctx, w, args.steps, args.warmup,
                                                       table=not args.no_stage_table)
    S, dt, kt = res["S"], res["dt"], res["kt"]
    copy_gbs = copy_bandwidth(torch, ctx.device) if not args.no_copy else None
    fill_gbs = fill_bandwidth(torch, ctx.device) if not args.no_copy else None

    # the same step recorded once into a HIP graph and replayed (the calls allocate nothing and never
    # synchronise): what a caller in a tight loop pays when launch overhead matters
    graph = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        g.replay()
        torch.cuda.synchronize()
        t0g = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        dtg = time.perf_counter() - t0g
        graph = {"ms_per_step": dtg / args.steps * 1e3, "value": dw.C * args.steps / dtg, "unit": "strategies/s"}
        del g

    timeline = None
    if args.timeline > 0:
        nsel = min(args.timeline, dw.C)
        sel = np.sort(np.random.default_rng(7).choice(dw.C, nsel, replace=False)).astype(np.int64)
        sizes = 2 * w.cand["pp"][sel].astype(np.int64) * w.cand["m"][sel]
        off = np.concatenate([[0], np.cumsum(sizes)])
        d_sel = torch.from_numpy(sel).to(ctx.device)
        d_off = torch.from_numpy(off[:-1].copy()).to(ctx.device)
        t_start = torch.empty(int(off[-1]), dtype=torch.int64, device=ctx.device)
        t_end = torch.empty_like(t_start)
        ar0 = torch.empty((nsel, 64), dtype=torch.int64, device=ctx.device)
        ar1 = torch.empty_like(ar0)
        ds.distsim_timeline(ctx, dw, ev, d_sel, d_off, t_start, t_end, ar0, ar1)      # warm-up
        torch.cuda.synchronize()
        ctx.timing_enable(True)
        for _ in range(5):
            ds.distsim_timeline(ctx, dw, ev, d_sel, d_off, t_start, t_end, ar0, ar1)
        torch.cuda.synchronize()
        t_idle = torch.empty_like(t_start)
        for _ in range(5):
            ds.distsim_bubbles(ctx, dw, ev, d_sel, d_off, t_start, t_end, t_idle)
        torch.cuda.synchronize()
        kt3 = ctx.timing_read()
        tl_ms, tl_n = kt3["k_timeline"]
        bb_ms, bb_n = kt3["k_bubbles"]
        ctx.timing_enable(False)
        tl_s = tl_ms / max(tl_n, 1) / 1e3
        tl_bytes = int(off[-1]) * 16 + nsel * 64 * 16
        timeline = {"candidates": int(nsel), "stage_tasks": int(off[-1]), "ms": tl_s * 1e3,
                    "stage_tasks_per_s": int(off[-1]) / tl_s, "bound": "hbm",
                    "achieved": tl_bytes / tl_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": tl_bytes / tl_s / 1e9 / HBM_PEAK_GBS}
        if fill_gbs:
            timeline["frac_of_measured_fill"] = tl_bytes / tl_s / 1e9 / fill_gbs
        gp_ms, gp_n = kt3["k_timeline_gpipe"]
        timeline["gpipe_kernel_ms"] = gp_ms / max(gp_n, 1)
        timeline["note"] = ("ms spans the packing of the selection, the level-sweep dump (k_timeline) and the closed-form "
                            "dump of the GPipe candidates (k_timeline_gpipe, also given on its own)")
        bb_s = bb_ms / max(bb_n, 1) / 1e3
        bb_bytes = int(off[-1]) * 24                       # start and predecessor's end in, idle time out
        timeline["bubbles"] = {"ms": bb_s * 1e3, "bound": "hbm", "achieved": bb_bytes / bb_s / 1e9,
                               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bb_bytes / bb_s / 1e9 / HBM_PEAK_GBS}
        del t_start, t_end, t_idle, ar0, ar1

    ingest = None
    if args.ingest > 0:
        from workloads import make_comm_profiles, make_operator_records
        n_rec = args.ingest
        rec = make_operator_records(n_rec, 50_000)
        d_rec = torch.from_numpy(rec).to(ctx.device)
        eid, rep, num, wsp = ds.alloc_dedup(ctx, n_rec, ctx.device)
        prof = [torch.from_numpy(x).to(ctx.device) for x in make_comm_profiles(n_rec)]
        elapsed = torch.empty(n_rec, dtype=torch.int64, device=ctx.device)
        ds.distsim_dedup_events(ctx, d_rec, eid, rep, num, wsp)                               # warm-up
        ds.distsim_comm_event_times(ctx, prof[0], prof[1], prof[2], prof[3], elapsed)
        torch.cuda.synchronize()
        ctx.timing_enable(True)
        for _ in range(5):
            ds.distsim_dedup_events(ctx, d_rec, eid, rep, num, wsp)
            ds.distsim_comm_event_times(ctx, prof[0], prof[1], prof[2], prof[3], elapsed)
        torch.cuda.synchronize()
        kt2 = ctx.timing_read()
        ctx.timing_enable(False)
        dd_s = kt2["k_dedup"][0] / max(kt2["k_dedup"][1], 1) / 1e3
        ct_s = kt2["k_comm_event_times"][0] / max(kt2["k_comm_event_times"][1], 1) / 1e3
        n_ev = int(num.item())
        dd_bytes = n_rec * (rec.shape[1] * 8 + 4) + n_ev * 4         # records in, event ids and representatives out
        ct_bytes = n_rec * (4 + 4 + 8 + 8 + 8)
        ingest = {"records": n_rec, "words": int(rec.shape[1]), "events": n_ev,
                  "dedup": {"ms": dd_s * 1e3, "records_per_s": n_rec / dd_s, "bound": "hbm",
                            "achieved": dd_bytes / dd_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": dd_bytes / dd_s / 1e9 / HBM_PEAK_GBS},
                  "comm_event_times": {"ms": ct_s * 1e3, "records_per_s": n_rec / ct_s, "bound": "hbm",
                                       "achieved": ct_bytes / ct_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": ct_bytes / ct_s / 1e9 / HBM_PEAK_GBS}}
        del d_rec, eid, rep, wsp, prof, elapsed

    search = None
    if args.search > 0:
        n_s = int(args.search)
        gen = torch.Generator(device=ctx.device)
        gen.manual_seed(2306084230 + 13)
        times = torch.randint(1 << 20, 1 << 50, (n_s,), dtype=torch.int64, device=ctx.device, generator=gen)
        times[::977] = torch.iinfo(torch.int64).max                       # candidates that are not valid
        wgt = torch.randint(1, 1 << 12, (n_s,), dtype=torch.int64, device=ctx.device, generator=gen)
        best_s, scr_s = ds.alloc_search(ctx, n_s)
        ds.distsim_search(ctx, times, n_s, best_s, scr_s)                  # warm-up
        torch.cuda.synchronize()
        lo = torch.min(times)
        first = int(torch.nonzero(times == lo)[0].item())
        ok = best_s.cpu().tolist() == [first, int(lo.item())]
        ctx.timing_enable(True)
        for _ in range(10):
            ds.distsim_search(ctx, times, n_s, best_s, scr_s)
        torch.cuda.synchronize()
        ms0, n0 = ctx.timing_read()["k_search"]
        for _ in range(10):
            ds.distsim_search(ctx, times, n_s, best_s, scr_s, weight=wgt, objective=1)
        torch.cuda.synchronize()
        ms1, n1 = ctx.timing_read()["k_search"]
        ctx.timing_enable(False)
        s0, s1 = ms0 / max(n0, 1) / 1e3, ms1 / max(n1, 1) / 1e3
        search = {"candidates": n_s, "matches_torch_min": bool(ok),
                  "min": {"ms": s0 * 1e3, "bound": "hbm", "achieved": n_s * 8 / s0 / 1e9, "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": n_s * 8 / s0 / 1e9 / HBM_PEAK_GBS},
                  "weighted": {"ms": s1 * 1e3, "bound": "hbm", "achieved": n_s * 16 / s1 / 1e9, "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": n_s * 16 / s1 / 1e9 / HBM_PEAK_GBS}}
        del times, wgt, best_s, scr_s

    variants = None
    if args.variants > 0:
        variants = time_variants(ds, ctx, w, min(args.variants, dw.C))

    C = dw.C
    tasks = res["tasks"]
    roofline, roofline_alu = sweep_rooflines(res, read_traffic(args.workload), copy_gbs, read_valu_instructions(args.workload))

    second = None
    if args.second and args.second != "none" and args.second != args.workload:
        w2 = make_workload(args.second)
        r2, bufs2 = measure(ds, torch, ctx, w2, max(args.steps // 2, 3), 2)
        hbm2, alu2 = sweep_rooflines(r2, read_traffic(args.second), copy_gbs)
        second = {"workload": f"{args.second}: {r2['C']} candidates, {r2['S']} stages, {r2['tasks']} stage-tasks",
                  "value": r2["C"] * max(args.steps // 2, 3) / r2["dt"], "unit": "strategies/s",
                  "ms_per_step": r2["dt"] / max(args.steps // 2, 3) * 1e3,
                  "events_per_s": r2["events"] * max(args.steps // 2, 3) / r2["dt"],
                  "stage_tasks_per_s": r2["tasks"] * max(args.steps // 2, 3) / r2["dt"],
                  "sweep_span_ms": r2["sim_avg_s"] * 1e3, "roofline_hbm_frac": hbm2["frac"], "roofline_alu_frac": alu2["frac"]}
        del bufs2

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        ncores = min(os.cpu_count() or 1, 16)
        ns = min(C, 100_000 if args.workload == "hetero64" else 20_000)
        idx = np.sort(np.random.default_rng(20230608).choice(C, ns, replace=False))
        ws = subset(w, idx)
        oracle.simulate(subset(w, idx[:64]), nthreads=ncores)          # page the library in
        t1 = time.perf_counter()
        ora = oracle.simulate(ws, nthreads=ncores)
        t_or = time.perf_counter() - t1
        n1 = min(ns, 10_000)                                            # and the rate of one thread
        t2 = time.perf_counter()
        oracle.simulate(subset(w, idx[:n1]), nthreads=1)
        t_1 = time.perf_counter() - t2
        cpu_baseline = {"value": ns / t_or, "unit": "strategies/s", "cores": ncores, "kind": "oracle",
                        "sample": f"{ns} seeded candidates of {args.workload}, {t_or:.2f} s wall",
                        "events_per_s": int(ora["num_events"].sum()) / t_or,
                        "one_thread": {"value": n1 / t_1, "sample": f"first {n1} of the same sample, {t_1:.2f} s"}}
        got = out.batch_ns[:C].cpu().numpy()[idx]
        parity = {"sampled": int(ns), "batch_ns_equal": bool(np.array_equal(got, ora["batch_ns"]))}

    line = {
        "metric": "candidate strategies simulated/sec", "value": C * args.steps / dt, "unit": "strategies/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {C} candidates, L={dw.L}, V={dw.V}, "
                               f"{w.cluster['num_devices']} simulated devices, {S} stages, {tasks} stage-tasks",
                   "candidates": C, "valid": res["valid"]},
        "events_per_s": res["events"] * args.steps / dt, "stage_tasks_per_s": tasks * args.steps / dt,
        "events_replicated_per_s": res["events_replicated"] * args.steps / dt,
        "events_note": "events_per_s counts the events on the pp distinct device timelines of every candidate; "
                       "events_replicated_per_s multiplies each candidate's count by tp x dp, the size of the full "
                       "timeline of Algorithm 1 and the data-parallel modelling step (never the headline); "
                       "events and stage-tasks are those of the simulated timelines: the kernels visit a GPipe "
                       "candidate's stage-tasks in closed form, not one by one (roofline_alu counts the visited ones)",
        "timing_note": "value / ms_per_step: `steps` steps with the library's per-kernel timers off; kernel_ms and "
                       "the rooflines: a second pass of the same steps with the timers on",
        "kernel_ms": {k: (v[0] / max(v[1], 1)) * (v[1] / args.steps) for k, v in kt.items()},
        "kernel_ms_note": "k_simulate is the span of the two sweep kernels, which run side by side "
                          "(k_simulate_gpipe on a stream of the library's context); the other entries are single kernels",
        "roofline": roofline, "roofline_alu": roofline_alu,
        "hbm_copy_measured_GBs": copy_gbs,
        "hbm_fill_measured_GBs": fill_gbs,
        "second_workload": second,
        "graph_replay": graph, "timeline": timeline, "ingest": ingest, "search": search, "variants": variants,
        "cpu_baseline": cpu_baseline, "parity": parity,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
