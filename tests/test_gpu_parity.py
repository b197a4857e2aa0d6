"""HIP path vs CPU oracle, element by element, through the C ABI.  Needs an MI355X."""
import os

import numpy as np
import pytest

from helpers import mk, mk_cluster, mk_costs
from workloads import Workload, make_workload, subset

pytestmark = pytest.mark.gpu

INT64_MAX = np.iinfo(np.int64).max
NT = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("name", ["tiny", "tiny_b", "gpt24", "gpt48"])
def test_full_parity_small_configs(H, oracle_mod, name):
    _say(f"[case] full parity {name}")
    w = make_workload(name)
    hip = H.run_hip(w)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    H.assert_same(hip, ora, what=name)
    assert (hip["status"] == 0).all()
    H.assert_same(H.run_hip(w, table=False, split=True), ora, what=name + ", GPipe launch")


def test_tiny_golden_numbers(H):
    _say("[case] tiny golden")
    costs = mk_costs([1_000_000] * 4, [2_025_000] * 4, act=[4 << 20] * 4)
    w = mk(costs, mk_cluster(2), [(1, 1, 2, 4, 1, [0, 2, 4]), (1, 1, 2, 4, 0, [0, 2, 4])])
    hip = H.run_hip(w)
    assert list(hip["batch_ns"]) == [30_353_884, 30_301_942]
    rows, _ = H.rows_of(hip, np.arange(2))
    assert list(hip["comp_busy_ns"][rows]) == [24_200_000] * 4
    assert list(hip["comm_busy_ns"][rows]) == [103_884] * 4
    assert list(hip["stage_tab"][4][rows]) == [25_971, 0, 25_971, 0]      # p2p after a forward
    assert list(hip["stage_tab"][5][rows]) == [0, 25_971, 0, 25_971]      # p2p after a backward
    assert list(hip["stage_layers"][rows]) == [0 | 2 << 8, 2 | 4 << 8] * 2


@pytest.mark.parametrize("name,nsample", [("gpt96", 6000), ("hetero64", 30000)])
def test_sampled_parity_full_size_launch(H, oracle_mod, name, nsample):
    """The full candidate list goes through the library in one call (the launch shape the
    benchmark times); a seeded sample plus the extreme shapes is checked one by one."""
    _say(f"[case] sampled parity {name}")
    w = make_workload(name)
    hip = H.run_hip(w)
    rng = np.random.default_rng(123)
    idx = set(rng.choice(w.C, nsample, replace=False).tolist())
    work = w.cand["pp"].astype(np.int64) * w.cand["m"]
    idx.update(np.argsort(work)[-200:].tolist())
    idx.update(np.argsort(work)[:200].tolist())
    idx.update(range(0, 64)); idx.update(range(w.C - 64, w.C))
    idx = np.asarray(sorted(idx))
    ora = H.oracle_with_table(oracle_mod, subset(w, idx), NT)
    H.assert_same(hip, ora, idx=idx, what=name)
    # properties that hold for every candidate at any size
    assert (hip["status"] == 0).all()
    rows, cnt = H.rows_of(hip, np.arange(w.C))
    assert np.array_equal(cnt, w.cand["pp"]) and len(np.unique(rows)) == len(rows)
    seg_max = np.maximum.reduceat(hip["comp_busy_ns"][rows], np.cumsum(cnt) - cnt)
    assert np.all(hip["batch_ns"] >= seg_max)
    # entries that belong to no candidate are zero
    free = np.ones(len(hip["comp_busy_ns"]), bool)
    free[rows] = False
    assert not hip["comp_busy_ns"][free].any() and not hip["comm_busy_ns"][free].any()
    assert not hip["stage_tab"][:, free].any()
    m, pp = w.cand["m"].astype(np.int64), w.cand["pp"].astype(np.int64)
    assert np.all(hip["num_events"] >= 2 * m * pp + 2 * m * (pp - 1))


@pytest.mark.parametrize("name", ["gpt96", "hetero64"])
def test_full_parity_largest_configs(H, oracle_mod, name):
    """Every candidate of the two largest configurations, in the launch shape the benchmark times
    (no stage table), against the oracle on all host threads."""
    _say(f"[case] full parity {name}")
    w = make_workload(name)
    hip = H.run_hip(w, table=False)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    H.assert_same(hip, ora, what=name + " (all candidates)")


def test_without_stage_table(H, oracle_mod):
    """stage_tab == NULL: nothing per-stage is written by event generation and simulate composes
    the stage events itself; results, statuses and event counts must be the same."""
    _say("[case] no stage table")
    for name in ("gpt24", "gpt48"):
        w = make_workload(name)
        H.assert_same(H.run_hip(w, table=False), H.oracle_with_table(oracle_mod, w, NT), what=name + " lazy")
    costs = mk_costs([10] * 4, [20] * 4, tps=(1,))
    rows = [(1, 1, 2, 4, 1, None), (1, 1, 2, 4, 1, [0, 0, 4]), (1, 1, 2, 4, 1, [0, 2, 3]), (1, 1, 2, 4, 0, [0, 1, 4]),
            (2, 1, 2, 4, 1, None)]
    w = mk(costs, mk_cluster(2), rows)
    hip = H.run_hip(w, table=False)
    H.assert_same(hip, H.oracle_with_table(oracle_mod, w), what="lazy invalid")
    assert list(hip["status"]) == [0, 1, 1, 0, 1]
    big = mk_costs([1 << 48] * 4, [1 << 48] * 4)
    w3 = mk(big, mk_cluster(2), [(1, 1, 2, 1, 1, None), (1, 1, 2, 4, 1, None)])
    hip = H.run_hip(w3, table=False)
    H.assert_same(hip, H.oracle_with_table(oracle_mod, w3), what="lazy range")
    assert list(hip["status"]) == [0, 2]


def test_blocking_p2p(H, oracle_mod):
    _say("[case] blocking p2p")
    for name in ("gpt24", "gpt48"):
        w = make_workload(name)
        cl = dict(w.cluster); cl["p2p_blocking"] = 1
        wb = Workload(name + "+blocking", w.costs, cl, w.cand)
        H.assert_same(H.run_hip(wb), H.oracle_with_table(oracle_mod, wb, NT), what=wb.name)
    w = make_workload("gpt96")
    rng = np.random.default_rng(5)
    idx = np.sort(rng.choice(w.C, 3000, replace=False))
    cl = dict(w.cluster); cl["p2p_blocking"] = 1
    wb = Workload("gpt96+blocking", w.costs, cl, subset(w, idx).cand)
    H.assert_same(H.run_hip(wb, table=False), H.oracle_with_table(oracle_mod, wb, NT), what=wb.name)


def test_serialised_links(H, oracle_mod):
    """p2p_blocking = 2: sends queue on their link.  Activations made large enough that the queueing
    changes batch times; all three schedules; the ragged hetero64 shapes; the timeline dump."""
    _say("[case] serialised links")
    for name in ("gpt24", "gpt48"):
        w = make_workload(name)
        costs = dict(w.costs); costs["act_bytes"] = w.costs["act_bytes"] * 40
        cand = {k: v.copy() for k, v in w.cand.items()}
        cand["schedule"] = (np.arange(len(cand["schedule"])) % 3).astype(np.uint8)
        free = Workload(name + "+big act", costs, w.cluster, cand)
        cl = dict(w.cluster); cl["p2p_blocking"] = 2
        ws = Workload(name + "+links", costs, cl, cand)
        ora = H.oracle_with_table(oracle_mod, ws, NT)
        base = H.oracle_with_table(oracle_mod, free, NT)
        ok = ora["status"] == 0
        assert np.all(ora["batch_ns"][ok] >= base["batch_ns"][ok]) and (ora["batch_ns"][ok] > base["batch_ns"][ok]).sum() > 50
        H.assert_same(H.run_hip(ws), ora, what=ws.name)
        H.assert_same(H.run_hip(ws, table=False), ora, what=ws.name + " no table")
    _timeline_parity(H, oracle_mod, ws, np.arange(2, ws.C, 11))
    w = make_workload("hetero64", C=30000)
    cl = dict(w.cluster); cl["p2p_blocking"] = 2
    costs = dict(w.costs); costs["act_bytes"] = w.costs["act_bytes"] * 25
    ws = Workload("hetero64+links", costs, cl, w.cand)
    H.assert_same(H.run_hip(ws, table=False), H.oracle_with_table(oracle_mod, ws, NT), what=ws.name)
    rng = np.random.default_rng(9)
    _timeline_parity(H, oracle_mod, ws, np.sort(rng.choice(ws.C, 60, replace=False)))


def _timeline_parity(H, oracle_mod, w, idx):
    import torch
    import paper_2306_08423_amd as ds
    c = H.ctx()
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, ds.stage_entries(w.cand["pp"]), table=False)
    ds.distsim_build_events(c, dw, ev)
    out = ds.alloc_outputs(c, ev)
    ds.distsim_simulate(c, dw, ev, out)
    idx = np.asarray(idx, np.int64)
    vch = np.ones(w.C, np.int64)                      # rows per device: chunks, or S / pp for explicit schedules (as a fraction)
    rows_of_c = w.cand["pp"].astype(np.int64).copy()  # rows of the dump: stages or virtual stages
    if w.cand.get("chunks") is not None:
        vch = np.where(w.cand["schedule"] == 3, w.cand["chunks"], 1).astype(np.int64)
        rows_of_c = rows_of_c * vch
        if w.cand.get("schedule_off") is not None:
            for cc in np.nonzero(w.cand["schedule"] == 4)[0]:
                sid = int(w.cand["chunks"][cc])
                if 0 <= sid < len(w.cand["schedule_off"]) - 1 and 0 <= int(w.cand["schedule_off"][sid]) < len(w.cand["schedule_words"]) - 1:
                    rows_of_c[cc] = int(w.cand["schedule_words"][int(w.cand["schedule_off"][sid]) + 1])
    sizes = 2 * rows_of_c[idx] * w.cand["m"][idx]
    off = np.concatenate([[0], np.cumsum(sizes)])
    dev = c.device
    start = torch.full((int(off[-1]),), -7, dtype=torch.int64, device=dev)
    end = torch.full((int(off[-1]),), -7, dtype=torch.int64, device=dev)
    ar0 = torch.full((len(idx), 64), -7, dtype=torch.int64, device=dev)
    ar1 = torch.full((len(idx), 64), -7, dtype=torch.int64, device=dev)
    ds.distsim_timeline(c, dw, ev, torch.from_numpy(idx).to(dev), torch.from_numpy(off[:-1].copy()).to(dev),
                        start, end, ar0, ar1)
    idle = torch.full((int(off[-1]),), -7, dtype=torch.int64, device=dev)
    ds.distsim_bubbles(c, dw, ev, torch.from_numpy(idx).to(dev), torch.from_numpy(off[:-1].copy()).to(dev), start, end, idle)
    torch.cuda.synchronize()
    start, end, ar0, ar1, idle = (t.cpu().numpy() for t in (start, end, ar0, ar1, idle))
    batch = out.batch_ns.cpu().numpy()
    from oracle.bubbles import idle_before
    hstat = ev.status.cpu().numpy()
    for k, i in enumerate(idx):
        r = oracle_mod.simulate(subset(w, [i]), timeline=True)
        pp, m = int(w.cand["pp"][i]), int(w.cand["m"][i])
        if r["status"][0] != 0 or hstat[i] == 4:                 # no strategy, or beyond the library: nothing is written
            assert (start[off[k]:off[k + 1]] == -7).all() and (ar0[k] == -1).all()
            assert (idle[off[k]:off[k + 1]] == -7).all()
            continue
        S = int(rows_of_c[i])                             # rows: stages, or virtual stages
        if int(w.cand["schedule"][i]) == 4:
            from oracle.bubbles import idle_before_lists
            from workloads.schedules import unpack_schedule
            sid = int(w.cand["chunks"][i])
            o0, o1 = int(w.cand["schedule_off"][sid]), int(w.cand["schedule_off"][sid + 1])
            lists = unpack_schedule(w.cand["schedule_words"][o0:o1])[5]
            want_idle = idle_before_lists(r["start"], r["end"], lists)
            listed = r["start"] >= 0
            got = idle[off[k]:off[k + 1]].reshape(2, S, m)
            assert np.array_equal(got[listed], want_idle[listed]) and (got[~listed] == -7).all(), (i, "idle")
            idle[off[k]:off[k + 1]] = want_idle.reshape(-1)          # checked; let the common line below pass
        else:
            want_idle = idle_before(r["start"], r["end"], int(w.cand["schedule"][i]), int(vch[i]))
        assert np.array_equal(idle[off[k]:off[k + 1]].reshape(2, S, m), want_idle), (i, "idle")
        assert np.array_equal(start[off[k]:off[k + 1]].reshape(2, S, m), r["start"]), (i, "start")
        assert np.array_equal(end[off[k]:off[k + 1]].reshape(2, S, m), r["end"]), (i, "end")
        assert np.array_equal(ar0[k, :pp], r["ar_window"][0]) and np.array_equal(ar1[k, :pp], r["ar_window"][1]), i
        assert (ar0[k, pp:] == -1).all() and (ar1[k, pp:] == -1).all()
        # the timeline ends where the simulation says the batch ends
        assert max(int(end[off[k]:off[k + 1]].max()), int(ar1[k].max())) == batch[i] == r["batch_ns"][0]


def test_timeline_dump(H, oracle_mod):
    _say("[case] timeline")
    w = make_workload("gpt24")
    _timeline_parity(H, oracle_mod, w, np.arange(0, w.C, 3))
    cl = dict(w.cluster); cl["p2p_blocking"] = 1
    _timeline_parity(H, oracle_mod, Workload("gpt24+blocking", w.costs, cl, w.cand), np.arange(1, w.C, 7))
    rng = np.random.default_rng(31)
    w = make_workload("gpt96")                                  # bucketed all-reduce windows
    _timeline_parity(H, oracle_mod, w, np.sort(rng.choice(w.C, 60, replace=False)))
    w = make_workload("hetero64", C=20000)
    _timeline_parity(H, oracle_mod, w, np.sort(rng.choice(w.C, 150, replace=False)))
    costs = mk_costs([10] * 4, [20] * 4)
    w = mk(costs, mk_cluster(2), [(1, 1, 2, 4, 1, None), (1, 1, 2, 4, 1, [0, 0, 4]), (2, 1, 2, 4, 1, None)])
    _timeline_parity(H, oracle_mod, w, [0, 1, 2])
    # indices outside the candidate list select nothing
    import torch
    import paper_2306_08423_amd as ds
    c = H.ctx()
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, ds.stage_entries(w.cand["pp"]), table=False)
    ds.distsim_build_events(c, dw, ev)
    out = ds.alloc_outputs(c, ev)
    ds.distsim_simulate(c, dw, ev, out)
    sel = torch.tensor([-1, 0, 3, 1 << 40], dtype=torch.int64, device=c.device)
    off = torch.tensor([0, 16, 32, 48], dtype=torch.int64, device=c.device)
    start = torch.full((64,), -7, dtype=torch.int64, device=c.device)
    end = torch.full((64,), -7, dtype=torch.int64, device=c.device)
    ar0 = torch.full((4, 64), -7, dtype=torch.int64, device=c.device)
    ar1 = torch.full((4, 64), -7, dtype=torch.int64, device=c.device)
    ds.distsim_timeline(c, dw, ev, sel, off, start, end, ar0, ar1)
    torch.cuda.synchronize()
    start = start.cpu().numpy()
    assert (start[:16] == -7).all() and (start[32:] == -7).all() and (start[16:32] >= 0).all()
    assert (ar0.cpu().numpy() == -1).all() and (ar1.cpu().numpy() == -1).all()


def test_async_schedule(H, oracle_mod):
    """Schedule 2 (Dapple order without the gradient all-reduce event) next to the other two, with and
    without buckets and the stage table, and in the timeline dump."""
    _say("[case] async schedule")
    w0 = make_workload("gpt48")
    rng = np.random.default_rng(12)
    cand = {k: v.copy() for k, v in w0.cand.items()}
    cand["schedule"] = rng.integers(0, 3, len(cand["schedule"])).astype(np.uint8)
    for bucket in (0, 25 << 20):
        cl = dict(w0.cluster); cl["dp_bucket_bytes"] = bucket
        w = Workload(f"gpt48+async bucket={bucket}", w0.costs, cl, cand)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        assert ((ora["status"] == 0) & (cand["schedule"] == 2)).sum() > 1000
        H.assert_same(H.run_hip(w), ora, what=w.name)
        H.assert_same(H.run_hip(w, table=False), ora, what=w.name + " no table")
    sel = np.nonzero(cand["schedule"] == 2)[0][::40]
    _timeline_parity(H, oracle_mod, w, sel)
    # an unknown schedule is an invalid candidate
    cand["schedule"][:5] = 5
    w = Workload("gpt48+bad schedule", w0.costs, w0.cluster, cand)
    hip = H.run_hip(w)
    assert (hip["status"][:5] == 1).all()
    H.assert_same(hip, H.oracle_with_table(oracle_mod, w, NT), what=w.name)


@pytest.mark.parametrize("split", [False, True, "schedules", "schedules, split"])
def test_graph_capture_and_replay(H, oracle_mod, split):
    """The three calls allocate nothing and never synchronise, so a caller can record them into a
    HIP graph; every replay (with eager work and synchronisation in between) must give the eager
    result.  split: with the second sweep kernel forked onto the context's stream and joined.
    schedules: a list with explicit schedules (compiled inside distsim_build_events, on the
    context's stream when split) and, in a second list, interleaved candidates."""
    import torch
    import paper_2306_08423_amd as ds
    _say(f"[case] graph capture split={split}")
    w = make_workload("gpt48")
    if isinstance(split, str):
        import bench
        ws = {name: wv for name, wv, _, _ in bench.variant_workloads(w, 600)}
        for name in ("explicit_lists", "interleaved_2_chunks"):
            _graph_replay_case(H, oracle_mod, ws[name], H.ctx_split() if "split" in split.split(", ")[1:] else H.ctx())
        return
    _graph_replay_case(H, oracle_mod, w, H.ctx_split() if split else H.ctx())


def _graph_replay_case(H, oracle_mod, w, c):
    import torch
    import paper_2306_08423_amd as ds
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, ds.stage_entries(w.cand["pp"]), table=False)
    out = ds.alloc_outputs(c, ev, util=True)
    best, scratch = ds.alloc_search(c, dw.C)

    def step():
        ds.distsim_build_events(c, dw, ev)
        ds.distsim_simulate(c, dw, ev, out)
        ds.distsim_search(c, out.batch_ns, dw.C, best, scratch)

    def results():
        # per-stage entries by candidate: where a candidate's block lies may differ between runs
        # (the order of candidates that share an ordering bin), what it holds may not
        rows, _ = ds.stage_rows(ev.status.cpu().numpy()[:dw.C], ev.stage_pos.cpu().numpy()[:dw.C], w.cand["pp"])
        rows = torch.as_tensor(rows, device=out.comp_busy_ns.device)
        return (out.batch_ns.clone(), out.comp_busy_ns[rows].clone(), out.comm_busy_ns[rows].clone(), best.clone())

    step()
    torch.cuda.synchronize()
    want = results()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        out.batch_ns.fill_(-3); out.comp_busy_ns.fill_(-3); out.comm_busy_ns.fill_(-3); best.fill_(-3)
        ev.status.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(results(), want):
            assert torch.equal(a, b), rep
        step()                                             # eager work between replays
        torch.cuda.synchronize()
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert np.array_equal(out.batch_ns.cpu().numpy()[:dw.C], ora["batch_ns"])


def test_interleaved_schedule(H, oracle_mod):
    """Schedule 3 (several model chunks per device) next to the other schedules: uniform and explicit
    partitions, blocking and latency p2p, invalid combinations, large pipelines."""
    _say("[case] interleaved schedule")
    w0 = make_workload("gpt48")                       # L = 48, 128 devices
    rng = np.random.default_rng(17)
    cand = {k: v.copy() for k, v in w0.cand.items()}
    C = len(cand["pp"])
    chunks = np.ones(C, np.int32)
    pick = rng.random(C) < 0.5
    cand["schedule"][pick] = 3
    chunks[pick] = rng.integers(1, 7, int(pick.sum()))
    cand["chunks"] = chunks
    for blocking in (0, 1, 2):
        cl = dict(w0.cluster); cl["p2p_blocking"] = blocking
        w = Workload(f"gpt48+interleaved blocking={blocking}", w0.costs, cl, cand)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        n_ok = int(((ora["status"] == 0) & (cand["schedule"] == 3)).sum())
        assert n_ok > 300
        hip = H.run_hip(w, table=False)
        H.assert_same(hip, ora, what=w.name)
        assert not (hip["status"] == 4).any()
        H.assert_same(H.run_hip(w), ora, what=w.name + " with table")
        # dump and bubbles, both kinds of candidates
        ok3 = np.nonzero((ora["status"] == 0) & (cand["schedule"] == 3))[0]
        sel = np.sort(np.concatenate([ok3[::max(1, len(ok3) // 40)], np.arange(0, C, 97)]))
        _timeline_parity(H, oracle_mod, w, np.unique(sel))
    # queues on the links that really delay: large activations
    big = dict(w0.costs); big["act_bytes"] = w0.costs["act_bytes"] * 40
    cl = dict(w0.cluster); cl["p2p_blocking"] = 2
    w = Workload("gpt48+interleaved, long transfers, link queues", big, cl, cand)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    free = oracle_mod.simulate(Workload("free", big, w0.cluster, cand), nthreads=NT)
    ok3 = (ora["status"] == 0) & (cand["schedule"] == 3)
    assert (ora["batch_ns"][ok3] > free["batch_ns"][ok3]).sum() > 100
    H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
    _timeline_parity(H, oracle_mod, w, np.nonzero(ok3)[0][::25])
    # bucketed all-reduce: a device fills its buckets across its chunks (results, all-reduce windows)
    for bucket, blocking in ((8 << 20, 0), (1 << 20, 1), (64 << 20, 2)):
        cl = dict(w0.cluster); cl["dp_bucket_bytes"] = bucket; cl["p2p_blocking"] = blocking
        w = Workload(f"gpt48+interleaved bucket={bucket} blocking={blocking}", w0.costs, cl, cand)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        plain = oracle_mod.simulate(Workload("trailing", w0.costs, dict(cl, dp_bucket_bytes=0), cand), nthreads=NT)
        ok3 = (ora["status"] == 0) & (cand["schedule"] == 3)
        assert (ora["num_events"][ok3] > plain["num_events"][ok3]).sum() > 100          # the buckets are events of their own
        H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
        _timeline_parity(H, oracle_mod, w, np.nonzero(ok3)[0][::20])
    # without chunk counts an interleaved candidate is invalid
    nc = {k: v for k, v in cand.items() if k != "chunks"}
    w = Workload("gpt48+interleaved no chunks", w0.costs, w0.cluster, nc)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert (ora["status"][pick] == 1).all()
    H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
    # explicit partitions into pp * chunks parts, ragged sizes, many micro-batches, 64 virtual stages
    L = 96
    costs = mk_costs(rng.integers(0, 5000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(0, 100, (2, L)) * 64).tolist(), grad=rng.integers(0, 1 << 20, (2, L)).tolist(),
                     a2a=(rng.integers(0, 3, (2, L)) * 4096).tolist(), tps=(1, 2))
    N = 64 * 9 * 5 * 7
    rows = []
    for pp, v in [(1, 1), (1, 5), (2, 2), (2, 32), (3, 4), (4, 16), (5, 3), (7, 9), (8, 8), (16, 4), (21, 3), (32, 2), (64, 1),
                  (9, 7), (12, 5), (6, 11)]:
        for tp in (1, 2):
            if N % (pp * tp):
                continue
            dp = N // (pp * tp)
            for groups in (1, 2, 5):
                S = pp * v
                bnd = None
                if S <= L and (pp + v + groups) % 2 == 0:
                    cuts = np.sort(rng.choice(np.arange(1, L), S - 1, replace=False))
                    bnd = [0] + cuts.tolist() + [L]
                rows.append((dp, tp, pp, pp * groups, 3, bnd, v))
    rows.append((N // 8, 1, 8, 8 * 40, 3, None, 8))                   # more slots than the ring holds
    rows.append((N // 2, 1, 2, 2 * 200, 3, None, 3))
    rows.append((N // 4, 1, 4, 6, 3, None, 2))                        # m not a multiple of pp
    rows.append((N // 4, 1, 4, 8, 3, [0, 10, 20, 30, 96], 2))         # too few boundaries in the pool (runs off its end)
    rows.append((N // 4, 1, 4, 8, 1, None))                           # a Dapple candidate among them
    rows.append((N // 12, 1, 12, 24, 3, None, 6))                     # 72 virtual stages: a strategy, but beyond this library
    rows.append((N // 12, 1, 12, 25, 3, None, 6))                     # the same with m not a multiple of pp: invalid
    w = mk(costs, mk_cluster(N), rows)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert (ora["status"] == 0).sum() > 40 and ora["status"][-2:].tolist() == [0, 1]
    hip = H.run_hip(w, table=False)
    assert hip["status"][-2:].tolist() == [4, 1]
    H.assert_same(hip, ora, what="interleaved ragged")
    _timeline_parity(H, oracle_mod, w, np.arange(0, w.C, 3))
    # many candidates of few devices and many chunks: the candidates that share a wavefront have more
    # virtual stages than its table holds, so it takes them in several passes
    rows = []
    for pp in (1, 2, 3, 4, 5, 8):
        for v in (6, 8, 12, 16, 21, 32, 64):
            if pp * v > 64:
                continue
            for groups in (1, 2, 3, 4, 7):
                rows.append((N // pp, 1, pp, pp * groups, 3, None, v))
    w = mk(costs, mk_cluster(N), rows)
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert (ora["status"] == 0).sum() > 100
    H.assert_same(H.run_hip(w, table=False), ora, what="interleaved, many chunks on few devices")
    _timeline_parity(H, oracle_mod, w, np.arange(0, w.C, 7))


def test_runs_are_deterministic(H):
    _say("[case] determinism")
    w = make_workload("gpt48")
    a, b = H.run_hip(w), H.run_hip(w)
    for k in ("status", "batch_ns", "num_events"):
        assert np.array_equal(a[k], b[k]), k
    # the order of equal-key candidates inside the library may differ between runs; what a
    # candidate's block holds may not
    ra, _ = H.rows_of(a, np.arange(w.C))
    rb, _ = H.rows_of(b, np.arange(w.C))
    for k in ("comp_busy_ns", "comm_busy_ns", "stage_layers"):
        assert np.array_equal(a[k][ra], b[k][rb]), k
    assert np.array_equal(a["stage_tab"][:, ra], b["stage_tab"][:, rb])
    assert a["util"][ra].tobytes() == b["util"][rb].tobytes()


def test_ragged_shapes_and_odd_stage_counts(H, oracle_mod):
    """pp that is not a power of two (idle lanes inside a group), pp = 64 with many
    micro-batches, m = 1, single stage, zero durations."""
    _say("[case] ragged shapes")
    rng = np.random.default_rng(77)
    L = 96
    costs = mk_costs(rng.integers(0, 5000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(0, 100, (2, L)) * 64).tolist(),
                     grad=rng.integers(0, 1 << 20, (2, L)).tolist(),
                     a2a=(rng.integers(0, 3, (2, L)) * 4096).tolist(), tps=(1, 2))
    rows = []
    N = 64 * 9 * 5 * 7 * 11                # 221 760: many divisors
    for pp in (1, 2, 3, 5, 6, 7, 9, 10, 11, 12, 14, 15, 18, 20, 21, 22, 24, 28, 30, 33, 35, 36, 42, 44, 45, 55,
               60, 63, 64, 66):
        for tp in (1, 2):
            if N % (pp * tp):
                continue
            dp = N // (pp * tp)
            for m in (1, 2, 3, 17, 64):
                for sc in (0, 1):
                    bnd = None
                    if pp <= L and (pp + m + sc) % 3 == 0:
                        cuts = np.sort(rng.choice(np.arange(1, L), pp - 1, replace=False))
                        bnd = [0] + cuts.tolist() + [L]
                    rows.append((dp, tp, pp, m, sc, bnd))
    rows.append((N // 64, 1, 64, 512, 1, None))
    rows.append((N // 64, 1, 64, 512, 0, None))
    for bucket in (0, 1 << 18):
        w = mk(costs, mk_cluster(N, bucket=bucket), rows)
        hip = H.run_hip(w)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        H.assert_same(hip, ora, what=f"ragged bucket={bucket}")
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"ragged bucket={bucket}, GPipe launch")
        assert (ora["status"] == 0).sum() > 200
    # all-zero table
    z = mk_costs([0] * 8, [0] * 8)
    w = mk(z, mk_cluster(4), [(1, 1, 4, 3, 1, None), (2, 1, 2, 1, 0, None), (4, 1, 1, 9, 0, None)])
    H.assert_same(H.run_hip(w), H.oracle_with_table(oracle_mod, w), what="zeros")


def test_gpipe_closed_form_items(H, oracle_mod):
    """GPipe candidates get their end times from the closed form of the recurrence, not from a sweep:
    in a kernel of their own, in pairs of wave-items (for long lists; the harness's second context
    does so for any list), and as lanes left out of the sweep elsewhere.  Items of one class that
    differ in pp and in m, odd numbers of GPipe items per class (the odd one goes the usual way), stage
    counts that are not powers of two, m = 1, other schedules next to them in one wave-item, all three
    readings of the p2p events, bucketed all-reduce, and per-stage arrays too small for all of them."""
    _say("[case] GPipe pairs")
    rng = np.random.default_rng(123)
    L = 80
    costs = mk_costs(rng.integers(0, 7000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 400, (2, L)).tolist(), ba=rng.integers(0, 400, (2, L)).tolist(),
                     act=(rng.integers(0, 200, (2, L)) * 128).tolist(), grad=rng.integers(0, 1 << 21, (2, L)).tolist(),
                     tps=(1, 2))
    N = 64 * 27 * 25 * 7 * 11
    divs = [p for p in range(1, 65) if N % p == 0]
    rows = []
    for rep in range(1500):
        pp = int(rng.choice(divs))
        tp = int(rng.choice([1, 2])) if (N // pp) % 2 == 0 else 1
        m = int(rng.choice([1, 2, 3, 5, 8, 13, 30, 31, 32, 33, 70]))
        sc = int(rng.choice([0, 0, 0, 1, 2]))
        bnd = None
        if rng.random() < 0.5:
            bnd = [0] + np.sort(rng.choice(np.arange(1, L), pp - 1, replace=False)).tolist() + [L]
        rows.append((N // (pp * tp), tp, pp, m, sc, bnd))
    for blocking, bucket in ((2, 0), (0, 0), (1, 0), (0, 1 << 19)):
        w = mk(costs, mk_cluster(N, blocking=blocking, bucket=bucket), rows)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        assert ((ora["status"] == 0) & (w.cand["schedule"] == 0)).sum() > 700
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"gpipe pairs blocking={blocking} bucket={bucket}")
        H.assert_same(H.run_hip(w, table=False), ora, what=f"one launch blocking={blocking} bucket={bucket}")
    H.assert_same(H.run_hip(w, split=True), ora, what="gpipe pairs with table")
    _timeline_parity(H, oracle_mod, w, np.arange(0, w.C, 29))
    # room for a part of the items only: the candidates that fit keep their results
    full = H.run_hip(w, table=False, split=True)
    need = int(full["stage_pos"].max()) + 64
    for cap in (need // 2, need // 3 + 64, 640, 64):
        part = H.run_hip(w, table=False, stage_cap=cap, split=True)
        fit = part["status"] == 0
        assert ((part["status"] == 3) | fit | (full["status"] != 0)).all() and fit.sum() > 0 and (part["status"] == 3).sum() > 0
        assert np.array_equal(part["batch_ns"][fit], full["batch_ns"][fit])
        assert np.array_equal(part["num_events"][fit], full["num_events"][fit])
        rp, _ = H.rows_of(part, np.nonzero(fit)[0])
        rf, _ = H.rows_of(full, np.nonzero(fit)[0])
        assert np.array_equal(part["comp_busy_ns"][rp], full["comp_busy_ns"][rf])
        assert np.array_equal(part["comm_busy_ns"][rp], full["comm_busy_ns"][rf])
        assert (part["batch_ns"][part["status"] == 3] == INT64_MAX).all()


def test_random_small_workloads(H, oracle_mod):
    """Seeded random tables, clusters and candidate lists of every kind the interface takes (all four
    schedules, the three p2p readings, buckets, several tensor-parallel variants, explicit and
    uniform partitions, invalid candidates in between), through both ways of launching."""
    _say("[case] random small workloads")
    rng = np.random.default_rng(20230608)
    for trial in range(24):
        L = int(rng.integers(1, 130))
        tps = [1] + sorted(rng.choice([2, 3, 4, 8], size=int(rng.integers(0, 3)), replace=False).tolist())
        V = len(tps)
        scale = int(rng.choice([1, 1000, 1 << 20, 1 << 34, 1 << 42]))
        costs = mk_costs((rng.integers(0, 7, (V, L)) * scale).tolist(), (rng.integers(0, 9, (V, L)) * scale).tolist(),
                         fa=(rng.integers(0, 3, (V, L)) * scale).tolist(), ba=(rng.integers(0, 3, (V, L)) * scale).tolist(),
                         act=(rng.integers(0, 50, (V, L)) * int(rng.choice([1, 4096, 1 << 24]))).tolist(),
                         grad=(rng.integers(0, 9, (V, L)) * int(rng.choice([1, 1 << 16, 1 << 26]))).tolist(),
                         a2a=(rng.integers(0, 2, (V, L)) * 8192).tolist(), tps=tuple(tps))
        N = int(rng.choice([1, 2, 6, 8, 24, 64, 360, 1024, 5040, 1 << 20]))
        blocking = int(rng.integers(0, 3))
        cl = mk_cluster(N, g=int(rng.choice([1, 2, 4, 8, 16])), alpha=(int(rng.integers(0, 9000)), int(rng.integers(0, 20000))),
                        beta=(int(rng.integers(1, 400)), int(rng.integers(1, 60))),
                        bucket=int(rng.choice([0, 0, 1 << 12, 1 << 22])), blocking=blocking)
        rows = []
        for _ in range(int(rng.integers(1, 260))):
            if rng.random() < 0.85:                               # a factorisation of the cluster
                pp = int(rng.choice([d for d in range(1, 65) if N % d == 0]))
                tp = int(rng.choice([t for t in tps if (N // pp) % t == 0]))
                dp = N // (pp * tp)
            else:                                                 # anything: 5 is no variant, pp may exceed 64
                tp, pp, dp = int(rng.choice(tps + [5])), int(rng.integers(1, 70)), int(rng.integers(1, 9))
            m = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 33, 100]))
            sc = int(rng.choice([0, 0, 1, 1, 2, 3, 4]))
            v = int(rng.integers(1, 4))
            S = pp * v if sc == 3 else pp
            bnd = None
            if rng.random() < 0.5 and 1 <= S <= L:
                bnd = [0] + np.sort(rng.choice(np.arange(1, L), S - 1, replace=False)).tolist() + [L]
                if rng.random() < 0.05:
                    bnd[int(rng.integers(0, len(bnd)))] = int(rng.integers(0, L + 1))      # most likely no partition any more
            if sc == 3 and rng.random() < 0.7:
                m = pp * int(rng.integers(1, 4))
            rows.append((dp, tp, pp, m, sc, bnd, v))
        w = mk(costs, cl, rows, name=f"random {trial}")
        ora = H.oracle_with_table(oracle_mod, w, NT)
        H.assert_same(H.run_hip(w), ora, what=f"random {trial}")
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"random {trial}, GPipe launch")
        ok = np.nonzero(ora["status"] == 0)[0]
        if len(ok):
            _timeline_parity(H, oracle_mod, w, ok[:: max(1, len(ok) // 6)])


def test_explicit_schedules(H, oracle_mod):
    """Schedule 4: device lists given by the caller.  The built-in schedules written out as lists,
    bidirectional pipelines, random schedules over random placements, malformed and unrunnable
    schedules, next to candidates of the other schedules; blocking and latency p2p."""
    _say("[case] explicit schedules")
    from test_explicit_schedule_pins import random_schedule
    from workloads.schedules import (bidirectional_lists, bidirectional_stages, chain, dapple_lists, gpipe_lists,
                                     interleaved_lists, interleaved_stages, pack_schedule, pack_schedules)
    rng = np.random.default_rng(404)
    L = 48
    costs = mk_costs(rng.integers(0, 5000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(0, 100, (2, L)) * 64).tolist(), grad=rng.integers(0, 1 << 20, (2, L)).tolist(),
                     a2a=(rng.integers(0, 3, (2, L)) * 4096).tolist(), tps=(1, 2))
    N = 64 * 9 * 5 * 7
    blocks, rows = [], []

    def add(blk, pp, m, tp=1, bnd=None):
        blocks.append(blk)
        rows.append((N // (pp * tp), tp, pp, m, 4, bnd, len(blocks) - 1))
    for pp in (1, 2, 3, 4, 6, 8, 12, 16, 32, 64):
        for m in (1, 2, 5, 16, 32):
            if pp * m > 2048 or N % pp:
                continue
            tp = 2 if (pp + m) % 3 == 0 else 1
            bnd = None
            if pp <= L and (pp + m) % 2 == 0:
                bnd = [0] + np.sort(rng.choice(np.arange(1, L), pp - 1, replace=False)).tolist() + [L]
            if pp > L:
                continue
            add(pack_schedule(pp, chain(pp), m, pp, 1, gpipe_lists(pp, m)), pp, m, tp, bnd)
            add(pack_schedule(pp, chain(pp), m, pp, 1, dapple_lists(pp, m)), pp, m, tp, bnd)
            rows.append((N // (pp * tp), tp, pp, m, 0, bnd, 0))            # the same two through the built-in schedules
            rows.append((N // (pp * tp), tp, pp, m, 1, bnd, 0))
            if pp >= 2 and pp % 2 == 0 and 2 * pp * m <= 2048:
                add(pack_schedule(pp, bidirectional_stages(pp), m, pp, 2, bidirectional_lists(pp, m)), pp, m, tp, bnd)
    for pp, v, g in [(2, 2, 1), (2, 8, 3), (4, 4, 2), (8, 2, 4), (3, 5, 2), (16, 3, 1)]:
        m = pp * g
        add(pack_schedule(pp, interleaved_stages(pp, v), m, pp * v, 1, interleaved_lists(pp, v, m)), pp, m)
        rows.append((N // pp, 1, pp, m, 3, None, v))
    for _ in range(60):                                                    # random placements and orders
        pp = int(rng.choice([d for d in range(1, 13) if N % d == 0]))
        S, m, nparts = int(rng.integers(1, 20)), int(rng.integers(1, 7)), int(rng.integers(1, 9))
        place, prev, lists = random_schedule(rng, pp, S, m)
        part = [int(rng.integers(0, nparts)) for _ in range(S)]
        bnd = [0] + np.sort(rng.choice(np.arange(1, L), nparts - 1, replace=False)).tolist() + [L] if rng.random() < 0.6 else None
        add(pack_schedule(pp, list(zip(place, part, prev)), m, nparts, int(rng.choice([1, 2, 3])), lists), pp, m, 1, bnd)
        if rng.random() < 0.3 and len(lists[0]) >= 2:                      # the same with two tasks of device 0 swapped
            sw = [list(x) for x in lists]
            i = int(rng.integers(0, len(sw[0]) - 1))
            sw[0][i], sw[0][i + 1] = sw[0][i + 1], sw[0][i]
            add(pack_schedule(pp, list(zip(place, part, prev)), m, nparts, 1, sw), pp, m, 1, bnd)
    # malformed blocks
    good = pack_schedule(2, chain(2), 2, 2, 1, dapple_lists(2, 2))
    lists = dapple_lists(2, 2)
    add(good, 2, 2)
    add(good, 2, 3)                                                        # m differs
    add(good[:-1], 2, 2)                                                   # too short
    add(pack_schedule(2, chain(2), 2, 2, 1, [lists[0] + [lists[0][0]], lists[1]]), 2, 2)          # a task twice
    add(pack_schedule(2, chain(2), 2, 2, 1, [lists[1], lists[0]]), 2, 2)                          # wrong device
    add(pack_schedule(2, [(0, 0, -1), (1, 1, 0), (1, 1, 0)], 2, 2, 1, lists), 2, 2)              # two stages after one
    add(pack_schedule(2, [(0, 0, -1), (1, 5, 0)], 2, 2, 1, lists), 2, 2)                          # part out of range
    add(pack_schedule(2, chain(2), 2, 2, 0, lists), 2, 2)                                         # replicas < 1
    add(pack_schedule(64, chain(64), 33, 64, 1, [[] for _ in range(64)]), 64, 33)                 # 64 * 33 slots: too many
    rows.append((N // 2, 1, 2, 2, 4, None, len(blocks) + 3))                                      # no such schedule
    rows.append((N // 2, 1, 2, 2, 4, None, -1))
    off, words = pack_schedules(blocks)
    for blocking in (0, 1, 2):
        w = mk(costs, mk_cluster(N, blocking=blocking), rows, name=f"explicit blocking={blocking}")
        w.cand["schedule_off"], w.cand["schedule_words"] = off, words
        ora = H.oracle_with_table(oracle_mod, w, NT)
        x = w.cand["schedule"] == 4
        assert (ora["status"][x] == 0).sum() > 150 and (ora["status"][x] == 1).sum() > 10
        hip = H.run_hip(w, table=False)
        H.assert_same(hip, ora, what=w.name)
        H.assert_same(H.run_hip(w, split=True), ora, what=w.name + ", table, GPipe launch")
    # bucketed all-reduce: a device fills its buckets across its stages (results, all-reduce windows)
    gmean = int(np.asarray(costs["grad_bytes"]).mean())
    for bucket, blocking in ((max(1, gmean // 2), 0), (max(1, 3 * gmean), 1), (max(1, gmean // 7), 2)):
        w = mk(costs, mk_cluster(N, blocking=blocking, bucket=bucket), rows, name=f"explicit bucket={bucket} blocking={blocking}")
        w.cand["schedule_off"], w.cand["schedule_words"] = off, words
        ora = H.oracle_with_table(oracle_mod, w, NT)
        wp = mk(costs, mk_cluster(N, blocking=blocking), rows)
        wp.cand["schedule_off"], wp.cand["schedule_words"] = off, words
        plain = oracle_mod.simulate(wp, nthreads=NT)
        x4 = (w.cand["schedule"] == 4) & (ora["status"] == 0)
        assert (ora["num_events"][x4] != plain["num_events"][x4]).sum() > 50
        H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
        _timeline_parity(H, oracle_mod, w, np.nonzero(x4)[0][::3])
    # without the tables an explicit candidate is invalid
    w = mk(costs, mk_cluster(N), rows[:8])
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert (ora["status"][w.cand["schedule"] == 4] == 1).all()
    H.assert_same(H.run_hip(w, table=False), ora, what="explicit without tables")
    # dump and bubbles of explicit candidates next to the others
    w = mk(costs, mk_cluster(N, blocking=1), rows, name="explicit dump")
    w.cand["schedule_off"], w.cand["schedule_words"] = off, words
    _timeline_parity(H, oracle_mod, w, np.arange(0, w.C, 2))
    # queues on the links that really delay: transfers much longer than the tasks
    long_act = dict(costs); long_act["act_bytes"] = costs["act_bytes"] * 400
    w = mk(long_act, mk_cluster(N, blocking=2), rows, name="explicit, long transfers, link queues")
    w.cand["schedule_off"], w.cand["schedule_words"] = off, words
    ora = H.oracle_with_table(oracle_mod, w, NT)
    wf = mk(long_act, mk_cluster(N), rows)
    wf.cand["schedule_off"], wf.cand["schedule_words"] = off, words
    free = oracle_mod.simulate(wf, nthreads=NT)
    x4 = (w.cand["schedule"] == 4) & (ora["status"] == 0)
    assert (ora["batch_ns"][x4] > free["batch_ns"][x4]).sum() > 50
    H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
    _timeline_parity(H, oracle_mod, w, np.arange(1, w.C, 3))


def test_explicit_schedules_without_a_program(H, oracle_mod):
    """Schedules that the library does not turn into a program and runs with the table of all task
    ends instead: a stage whose ends pile up (its consumer's device is busy with another pipeline
    first: more than 16 ends wait), blocks that lie beyond the first 2^17 words of the schedule array;
    next to schedules that do get a program.  And the order of the checks: lists that cannot be run to
    their ends are no strategy, but a candidate's own range check comes first."""
    _say("[case] explicit schedules without a program")
    from workloads.schedules import chain, dapple_lists, gpipe_lists, pack_schedule, pack_schedules
    rng = np.random.default_rng(77)
    L = 48
    costs = mk_costs(rng.integers(1, 5000, (2, L)).tolist(), rng.integers(1, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(1, 100, (2, L)) * 64).tolist(), grad=rng.integers(1, 1 << 20, (2, L)).tolist(),
                     tps=(1, 2))
    N = 64 * 9
    blocks, rows = [], []

    def add(blk, pp, m, tp=1, bnd=None):
        blocks.append(blk)
        rows.append((N // (pp * tp), tp, pp, m, 4, bnd, len(blocks) - 1))
    # stage 0 (device 0) feeds stage 1 (device 1), which starts only after device 1 has run all of
    # stage 2, a pipeline of its own
    for m in (3, 17, 40, 200):
        stages = [(0, 0, -1), (1, 1, 0), (1, 2, -1)]
        dev0 = [(0, 0, j) for j in range(m)] + [(1, 0, j) for j in range(m)]
        dev1 = [(0, 2, j) for j in range(m)] + [(1, 2, j) for j in range(m)] + [(0, 1, j) for j in range(m)] + [(1, 1, j) for j in range(m)]
        add(pack_schedule(2, stages, m, 3, 1, [dev0, dev1]), 2, m, 1, [0, 10, 30, L])
        add(pack_schedule(2, stages, m, 3, 2, [dev0, dev1]), 2, m, 2, None)
    # enough large blocks to pass 2^17 words; candidates on every one of them
    for q in range(36):
        pp, m = (16, 128) if q % 2 == 0 else (8, 256)
        lists = gpipe_lists(pp, m) if q % 3 == 0 else dapple_lists(pp, m)
        add(pack_schedule(pp, chain(pp), m, pp, 1, lists), pp, m, 1 + q % 2)
    off, words = pack_schedules(blocks)
    assert off[-1] > (1 << 17) + 8000 and off[8 + 20] < (1 << 17)
    # lists that cannot be run (device 1 wants stage 1's backward first), also with times out of range
    stuck = pack_schedule(2, chain(2), 2, 2, 1, [dapple_lists(2, 2)[0], dapple_lists(2, 2)[1][::-1]])
    blocks.append(stuck)
    rows.append((N // 2, 1, 2, 2, 4, None, len(blocks) - 1))
    off, words = pack_schedules(blocks)
    # two more entries of the offset table that point nowhere (sums of such offsets would wrap)
    off = np.concatenate([off, np.array([1 << 62, -5], dtype=np.int64)])
    rows.append((N // 2, 1, 2, 2, 4, None, len(blocks)))
    rows.append((N // 2, 1, 2, 2, 4, None, len(blocks) + 1))
    for blocking, bucket in ((0, 0), (2, 0), (1, 1 << 20)):
        w = mk(costs, mk_cluster(N, blocking=blocking, bucket=bucket), rows, name=f"no program, blocking={blocking} bucket={bucket}")
        w.cand["schedule_off"], w.cand["schedule_words"] = off, words
        ora = H.oracle_with_table(oracle_mod, w, NT)
        assert (ora["status"][:-3] == 0).all() and (ora["status"][-3:] == 1).all()
        H.assert_same(H.run_hip(w, table=False), ora, what=w.name)
        _timeline_parity(H, oracle_mod, w, np.arange(0, w.C - 3, 5))
    huge = dict(costs); huge["fwd_comp_ns"] = costs["fwd_comp_ns"] * (1 << 40)
    w = mk(huge, mk_cluster(N), rows[:4] + rows[-3:-2], name="no program, out of range")
    w.cand["schedule_off"], w.cand["schedule_words"] = off, words
    ora = H.oracle_with_table(oracle_mod, w, NT)
    assert (ora["status"] == 2).all()
    H.assert_same(H.run_hip(w, table=False), ora, what=w.name)


def test_bench_variants_parity(H, oracle_mod):
    """The variant workloads that bench.py times (other p2p readings, asynchronous, interleaved and
    explicit schedules on a seeded sample of hetero64), in the launch shapes of the benchmark: every
    group of every wavefront of the interleaved and the explicit kernels is filled."""
    _say("[case] bench variants")
    import bench
    w0 = make_workload("hetero64")
    for name, wv, kernel, counted in bench.variant_workloads(w0, 20000):
        ora = oracle_mod.simulate(wv, nthreads=NT)
        assert (ora["status"][counted] == 0).all(), name
        H.assert_same(H.run_hip(wv, table=False), ora, what="bench variant " + name)


def test_uniform_partition_every_shape(H, oracle_mod):
    """The uniform partition rule floor(s L / pp) for every layer count 1..255 and every stage count
    it admits (up to 64), through the level sweeps and, with 2 and 3 chunks, the interleaved kernel."""
    _say("[case] uniform partitions, every (L, pp)")
    rng = np.random.default_rng(9)
    n = 0
    for L in range(1, 256):
        costs = mk_costs(rng.integers(1, 1000, (1, L)).tolist(), rng.integers(1, 1000, (1, L)).tolist(),
                         act=(rng.integers(1, 9, (1, L)) * 64).tolist(), grad=rng.integers(1, 99, (1, L)).tolist())
        for pp in range(1, min(L, 64) + 1):
            rows = [(1, 1, pp, 3, 1, None), (1, 1, pp, 2, 0, None)]
            rows += [(1, 1, pp, pp, 3, None, v) for v in (2, 3) if pp * v <= min(L, 64)]
            w = mk(costs, mk_cluster(pp), rows)
            ora = H.oracle_with_table(oracle_mod, w)
            assert (ora["status"] == 0).all(), (L, pp)
            H.assert_same(H.run_hip(w, table=(pp % 7 == 0)), ora, what=f"uniform L={L} pp={pp}")
            n += 1
    assert n == 14304


def test_maximum_micro_batch_count(H, oracle_mod):
    """The largest micro-batch count the interface takes (2^16) with the deepest pipeline (64
    stages, 131 198 levels), with few stages and with one; every schedule of the level sweeps; one
    more micro-batch is invalid.  Also blocking p2p, buckets, the serialised links and the dump of
    a candidate of 655 360 stage-tasks."""
    _say("[case] maximum micro-batch count")
    rng = np.random.default_rng(3)
    L = 96
    costs = mk_costs(rng.integers(0, 5000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(0, 100, (2, L)) * 64).tolist(), grad=rng.integers(0, 1 << 20, (2, L)).tolist(),
                     tps=(1, 2))
    N, M = 64 * 15, 1 << 16
    rows = [(N // 64, 1, 64, M, 0, None), (N // 64, 1, 64, M, 1, None), (N // 64, 1, 64, M, 2, None),
            (N // 10, 2, 5, M, 1, None), (N, 1, 1, M, 0, None), (N // 64, 1, 64, M + 1, 1, None),
            (N // 3, 1, 3, M - 1, 0, None), (N // 64, 1, 64, M, 0, None)]
    for blocking, bucket in ((0, 0), (1, 1 << 18), (2, 0)):
        w = mk(costs, mk_cluster(N, blocking=blocking, bucket=bucket), rows)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        assert ora["status"].tolist() == [0] * 8             # the method has no bound on m ...
        hip = H.run_hip(w)
        assert hip["status"].tolist() == [0, 0, 0, 0, 0, 4, 0, 0]      # ... the library has, and says so
        H.assert_same(hip, ora, what=f"m = 2^16, blocking={blocking} bucket={bucket}")
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"m = 2^16, blocking={blocking}, GPipe launch")
    w = mk(costs, mk_cluster(N), rows)
    _timeline_parity(H, oracle_mod, w, [3])


def test_invalid_range_and_capacity_status(H, oracle_mod):
    _say("[case] status codes")
    costs = mk_costs([10] * 4, [20] * 4, tps=(1,))
    rows = [
        (1, 1, 2, 4, 1, None), (2, 1, 2, 4, 1, None), (1, 2, 1, 4, 1, None), (1, 1, 2, 0, 1, None),
        (1, 1, 2, 4, 1, [0, 0, 4]), (1, 1, 2, 4, 1, [0, 2, 3]), (1, 1, 2, 4, 5, None), (1, 1, 2, 4, 0, [0, 1, 4]),
        (1, 1, 2, (1 << 16) + 1, 0, None), (-1, -1, 2, 4, 0, None), (1, 1, 0, 4, 0, None),
    ]
    w = mk(costs, mk_cluster(2), rows)
    hip, ora = H.run_hip(w), H.oracle_with_table(oracle_mod, w)
    H.assert_same(hip, ora, what="invalid mix")
    assert list(hip["status"]) == [0, 1, 1, 1, 1, 1, 1, 0, 4, 1, 1]
    assert all(hip["batch_ns"][i] == INT64_MAX for i in (1, 2, 3, 4, 5, 6, 8, 9, 10))
    # partition offsets outside the pool
    w2 = mk(costs, mk_cluster(2), [(1, 1, 2, 4, 1, [0, 2, 4])])
    w2.cand["part_off"][0] = 1
    assert H.run_hip(w2)["status"][0] == 1
    w2.cand["part_off"][0] = -5
    assert H.run_hip(w2)["status"][0] == 1
    # 2^53 guard
    big = mk_costs([1 << 48] * 4, [1 << 48] * 4)
    w3 = mk(big, mk_cluster(2), [(1, 1, 2, 1, 1, None), (1, 1, 2, 4, 1, None), (1, 1, 2, 3, 0, None), (1, 1, 2, 5, 0, None)])
    hip, ora = H.run_hip(w3), H.oracle_with_table(oracle_mod, w3)
    H.assert_same(hip, ora, what="range")
    assert list(hip["status"]) == [0, 2, 0, 2]
    # not enough room: candidates whose block does not fit are flagged, the others are untouched
    wide = mk_costs([10] * 64, [20] * 64)
    w4 = mk(wide, mk_cluster(40), [(1, 1, 40, 3, 1, None)] * 3)       # one 64-entry block each
    hip = H.run_hip(w4, stage_cap=130)
    assert sorted(hip["status"]) == [0, 0, 3]
    full = H.run_hip(w4)
    assert (full["status"] == 0).all()
    for i in range(3):
        if hip["status"][i] == 0:
            assert hip["batch_ns"][i] == full["batch_ns"][i]
            assert 0 <= hip["stage_pos"][i] <= 64
        else:
            assert hip["batch_ns"][i] == INT64_MAX and hip["stage_pos"][i] == -1 and hip["num_events"][i] == 0
    assert H.run_hip(w4, stage_cap=0)["status"].tolist() == [3, 3, 3]


def test_batch_ends_at_and_above_two_to_the_52(H, oracle_mod):
    """With one trailing all-reduce event the kernels keep the end of the batch in fp64 as long as every
    stage's end + event stays below 2^52 and take integers otherwise: ends between 2^52 and 2^53, events
    that push the sum past 2^53 (odd sums there have no double), and small candidates beside them."""
    _say("[case] batch ends at and above 2^52")
    for sched in (0, 1, 2):
        # pp = 2, m = 1: the first stage ends at 16 * 2^48 + 3 = 2^52 + 3
        costs = mk_costs([3 << 48, (3 << 48) + 1, 3 << 48, 3 << 48], [1 << 48, 1 << 48, (1 << 48) + 2, 1 << 48],
                         grad=[(1 << 52) + 1, 5, 1 << 40, 7], act=[0] * 4)
        cl = mk_cluster(4, g=8, alpha=(0, 0), beta=(1, 1))
        rows = [(2, 1, 2, 1, sched, [0, 2, 4]), (2, 1, 2, 1, sched, [0, 1, 4]), (4, 1, 1, 1, sched, None),
                (2, 1, 2, 1, sched, [0, 3, 4])]
        w = mk(costs, cl, rows)
        hip, ora = H.run_hip(w), H.oracle_with_table(oracle_mod, w)
        assert (ora["status"] == 0).all() and (ora["batch_ns"] >= 1 << 52).all()
        assert (ora["batch_ns"] % 2 == 1).any() and (sched == 2 or ((ora["batch_ns"] > 1 << 53) & (ora["batch_ns"] % 2 == 1)).any())
        H.assert_same(hip, ora, what=f"ends above 2^52, schedule {sched}")
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"ends above 2^52, schedule {sched}, two launches")
    # small and large candidates in one list (they share wavefronts of their class)
    small = mk_costs([3, 4, 5, 6], [7, 8, 9, 10], grad=[1 << 52, 1, 1, 1], act=[0] * 4)
    rows = [(2, 1, 2, m, sc, [0, 2, 4]) for m in (1, 2, 5) for sc in (0, 1)] + [(4, 1, 1, 3, 1, None)]
    w = mk(small, mk_cluster(4, g=8, alpha=(0, 0), beta=(1, 1)), rows)
    hip, ora = H.run_hip(w), H.oracle_with_table(oracle_mod, w)
    assert (ora["status"] == 0).all() and (ora["batch_ns"] > 1 << 51).any()
    H.assert_same(hip, ora, what="huge trailing events on short pipelines")


def test_warm_up_shapes_of_the_early_backward_schedules(H, oracle_mod):
    """The warm-up forwards of 1F1B and of the asynchronous schedule come from a closed form and the
    sweep starts at the first backward: every relation of m to pp (m = 1, m < pp, m = pp, m = pp + 1,
    m >> pp), stage counts that are not powers of two, all three readings of the p2p events, GPipe
    candidates beside them, both ways of launching."""
    _say("[case] warm-up shapes")
    rng = np.random.default_rng(77)
    L = 72
    costs = mk_costs(rng.integers(1, 5000, (2, L)).tolist(), rng.integers(1, 9000, (2, L)).tolist(),
                     fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                     act=(rng.integers(0, 300, (2, L)) * 200).tolist(), grad=rng.integers(0, 1 << 20, (2, L)).tolist(),
                     tps=(1, 2))
    N = 64 * 27 * 25 * 7 * 11
    rows = []
    for pp in (1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 48, 63, 64):
        if N % pp:
            continue
        for m in sorted({1, 2, max(1, pp - 1), pp, pp + 1, 2 * pp + 3, 150}):
            for sc in (1, 2, 0):
                bnd = [0] + np.sort(rng.choice(np.arange(1, L), pp - 1, replace=False)).tolist() + [L]
                rows.append((N // pp, 1, pp, m, sc, bnd))
    # strategies that event generation rejects, in between: the launch that runs beside k_simulate marks them
    nbad = 0
    for at in (3, 40, 41, len(rows) - 1):
        rows.insert(at, (7, 1, 5, 4, 1, None))          # dp tp pp is not the number of devices
        nbad += 1
    for blocking in (0, 1, 2):
        w = mk(costs, mk_cluster(N, blocking=blocking), rows)
        ora = H.oracle_with_table(oracle_mod, w, NT)
        assert (ora["status"] != 0).sum() == nbad and (ora["batch_ns"][ora["status"] != 0] == INT64_MAX).all()
        H.assert_same(H.run_hip(w, table=False), ora, what=f"warm-up shapes blocking={blocking}")
        H.assert_same(H.run_hip(w, table=False, split=True), ora, what=f"warm-up shapes blocking={blocking}, two launches")


def test_empty_candidate_list(H):
    _say("[case] C = 0")
    w = mk(mk_costs([1, 2], [3, 4]), mk_cluster(2), [])
    hip = H.run_hip(w, search=(0, None))
    assert hip["best"] == (-1, INT64_MAX)


def test_search_parity(H, oracle_mod):
    _say("[case] search")
    w = make_workload("gpt48")
    wgt = (w.cand["dp"].astype(np.int64) * w.cand["m"])
    for obj in (0, 1):
        hip = H.run_hip(w, search=(obj, wgt if obj else None))
        want = oracle_mod.search(hip["batch_ns"], wgt if obj else None, obj)
        assert hip["best"] == want
    # ties, invalid entries and all-invalid, on raw arrays
    import torch
    import paper_2306_08423_amd as ds
    c = H.ctx()
    rng = np.random.default_rng(8)
    for n in (1, 2, 63, 64, 65, 1000, 4097, 300_000, 3_000_001):        # the last: several turns of the grid's loop
        b = rng.integers(1, 1 << 52, n)
        b[rng.integers(0, n, n // 3 + 1)] = b[n // 2]
        b[rng.random(n) < 0.1] = INT64_MAX
        wg = rng.integers(-2, 1 << 20, n)
        for obj in (0, 1):
            best, scratch = ds.alloc_search(c, n)
            ds.distsim_search(c, torch.from_numpy(b).to(c.device), n, best, scratch,
                              weight=torch.from_numpy(wg).to(c.device), objective=obj)
            got = tuple(int(x) for x in best.cpu().numpy())
            assert got == oracle_mod.search(b, wg, obj), (n, obj)
    b = np.full(100, INT64_MAX)
    best, scratch = ds.alloc_search(c, 100)
    ds.distsim_search(c, torch.from_numpy(b).to(c.device), 100, best, scratch)
    assert tuple(int(x) for x in best.cpu().numpy()) == (-1, INT64_MAX)


def test_events_hold_nothing_of_the_callers_inputs(H, oracle_mod):
    """After distsim_build_events the cost table may go: simulate and the dump find what they need in
    the workspace and take the candidates as an argument.  Also the arrays of distsim_events carved
    out of one allocation (distsim_events_bytes / distsim_events_bind)."""
    import torch
    import paper_2306_08423_amd as ds
    _say("[case] events without the caller's inputs, one allocation")
    w = make_workload("gpt48")
    c = H.ctx()
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events_bound(c, dw, ds.stage_entries(w.cand["pp"]), table=True)
    ds.distsim_build_events(c, dw, ev)
    torch.cuda.synchronize()
    for k, t in dw.costs.items():                      # the table is gone (overwritten in place)
        t.fill_(-12345)
    torch.cuda.synchronize()
    out = ds.alloc_outputs(c, ev)
    ds.distsim_simulate(c, dw, ev, out)
    torch.cuda.synchronize()
    ora = H.oracle_with_table(oracle_mod, w, NT)
    hip = {"status": ev.status.cpu().numpy()[:dw.C], "num_events": ev.num_events.cpu().numpy()[:dw.C],
           "stage_pos": ev.stage_pos.cpu().numpy()[:dw.C], "batch_ns": out.batch_ns.cpu().numpy()[:dw.C],
           "comp_busy_ns": out.comp_busy_ns.cpu().numpy(), "comm_busy_ns": out.comm_busy_ns.cpu().numpy(),
           "util": out.util.cpu().numpy(), "pp": w.cand["pp"].astype(np.int64), "workload": w,
           "stage_tab": ev.stage_tab.cpu().numpy(), "stage_layers": ev.stage_layers.cpu().numpy()}
    H.assert_same(hip, ora, what="bound events, cost table released")
    # the dump as well (it looks up the tensor-parallel variant of a candidate)
    idx = np.arange(0, dw.C, 97, dtype=np.int64)
    sizes = 2 * w.cand["pp"][idx].astype(np.int64) * w.cand["m"][idx]
    off = np.concatenate([[0], np.cumsum(sizes)])
    start = torch.full((int(off[-1]),), -7, dtype=torch.int64, device=c.device)
    end = torch.full_like(start, -7)
    ar0 = torch.full((len(idx), 64), -7, dtype=torch.int64, device=c.device)
    ar1 = torch.full_like(ar0, -7)
    ds.distsim_timeline(c, dw, ev, torch.from_numpy(idx).to(c.device), torch.from_numpy(off[:-1].copy()).to(c.device),
                        start, end, ar0, ar1)
    torch.cuda.synchronize()
    end = end.cpu().numpy()
    for k, i in enumerate(idx):
        assert max(int(end[off[k]:off[k + 1]].max()), int(ar1[k].max().item())) == ora["batch_ns"][i]


def test_simulate_rejects_other_candidate_count(H):
    import paper_2306_08423_amd as ds
    w = make_workload("gpt24")
    c = H.ctx()
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, ds.stage_entries(w.cand["pp"]), table=False)
    ds.distsim_build_events(c, dw, ev)
    out = ds.alloc_outputs(c, ev)
    ev.C = dw.C - 1
    with pytest.raises(ds.DistSimError):
        ds.distsim_simulate(c, dw, ev, out)


def test_api_errors(H):
    _say("[case] api errors")
    import paper_2306_08423_amd as ds
    c = H.ctx()
    w = make_workload("tiny")
    dw = ds.upload(w, c.device)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, 4)
    ev.struct.workspace_bytes = 16
    with pytest.raises(ds.DistSimError, match="workspace too small"):
        ds.distsim_build_events(c, dw, ev)
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, 4)
    dw.cluster["beta_bytes_per_ns"] = (0, 25)
    with pytest.raises(ds.DistSimError, match="cluster"):
        ds.distsim_build_events(c, dw, ev)
    assert c.lib.distsim_workspace_bytes(300, 1, 10) == 0
