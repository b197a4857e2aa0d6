"""Pins of the oracle's explicit-schedule routine (schedule 4: the device lists of Algorithm 1's
schedule S given by the caller, Sec. 4.3).  CPU only.

 * the lists of GPipe, Dapple and the interleaved schedule, written out from their definitions
   (workloads/schedules.py), must give what the oracle's own routines for those schedules give:
   three routines, one answer;
 * random schedules (random placement of the stages on the devices, several pipelines, random
   subsets of the micro-batches, a random linear extension as execution order) against the longest
   path in the explicit task graph;
 * what makes a schedule invalid.
"""
import numpy as np
import pytest

from helpers import mk, mk_cluster, mk_costs
from workloads.schedules import (BWD, FWD, bidirectional_lists, bidirectional_stages, chain, dapple_lists,
                                 gpipe_lists, interleaved_lists, interleaved_stages, pack_schedule, pack_schedules)

INT64_MAX = (1 << 63) - 1


def with_schedules(w, blocks, ids):
    off, words = pack_schedules(blocks)
    w.cand["schedule_off"], w.cand["schedule_words"] = off, words
    w.cand["chunks"] = np.asarray(ids, np.int32)
    return w


def rand_costs(rng, L, tps=(1,)):
    V = len(tps)
    return mk_costs(rng.integers(0, 50, (V, L)).tolist(), rng.integers(0, 80, (V, L)).tolist(),
                    fa=rng.integers(0, 9, (V, L)).tolist(), ba=rng.integers(0, 9, (V, L)).tolist(),
                    act=(rng.integers(0, 9, (V, L)) * 5).tolist(), grad=rng.integers(0, 300, (V, L)).tolist(), tps=tps)


def same_result(a, b, ia, ib, what):
    for k in ("status", "batch_ns", "num_events"):
        assert a[k][ia] == b[k][ib], (what, k, a[k][ia], b[k][ib])
    sa, sb = a["stage_off"], b["stage_off"]
    for k in ("comp_busy_ns", "comm_busy_ns"):
        assert np.array_equal(a[k][sa[ia]:sa[ia + 1]], b[k][sb[ib]:sb[ib + 1]]), (what, k)


def test_builtin_schedules_written_out_as_lists(oracle_mod):
    rng = np.random.default_rng(5)
    for trial in range(180):
        pp = int(rng.integers(1, 7))
        v = int(rng.integers(1, 4))
        m = pp * int(rng.integers(1, 4)) if trial % 3 == 2 else int(rng.integers(1, 9))
        tp = int(rng.choice([1, 2]))
        dp = int(rng.choice([1, 2, 3]))
        L = pp * v + int(rng.integers(0, 5))
        costs = rand_costs(rng, L, tps=(1, 2))
        blocking = int(rng.integers(0, 3))          # latency on the edge, send on the device, sends queue on their link
        cl = mk_cluster(dp * tp * pp, g=int(rng.choice([1, 2, 4, 64])), alpha=(3, 11), beta=(5, 2), blocking=blocking)
        if blocking == 2:                           # transfers long enough to queue
            costs["act_bytes"] = costs["act_bytes"] * 20
        if trial % 3 == 2:                          # interleaved
            S = pp * v
            bnd = [0] + sorted(rng.choice(np.arange(1, L), S - 1, replace=False).tolist()) + [L]
            blk = pack_schedule(pp, interleaved_stages(pp, v), m, S, 1, interleaved_lists(pp, v, m))
            rows = [(dp, tp, pp, m, 3, bnd, v), (dp, tp, pp, m, 4, bnd, 0)]
        else:
            sched = trial % 3
            bnd = [0] + sorted(rng.choice(np.arange(1, L), pp - 1, replace=False).tolist()) + [L] if rng.random() < 0.7 else None
            lists = gpipe_lists(pp, m) if sched == 0 else dapple_lists(pp, m)
            blk = pack_schedule(pp, chain(pp), m, pp, 1, lists)
            rows = [(dp, tp, pp, m, sched, bnd, 1), (dp, tp, pp, m, 4, bnd, 0)]
        w = with_schedules(mk(costs, cl, rows), [blk], [r[6] for r in rows])
        r = oracle_mod.simulate(w)
        assert r["status"][0] == 0
        same_result(r, r, 0, 1, f"trial {trial}")


def longest_path(S, m, place, prev, lists, Fd, Bd, pf, pb, blocking):
    """End of every listed task by relaxation over the explicit graph: device order, the edge from
    the stage before (forward) or after (backward), the turn-around on a stage without successor."""
    nxt = {prev[k]: k for k in range(S) if prev[k] >= 0}
    preds = {}
    for lst in lists:
        for i, (kd, k, j) in enumerate(lst):
            p = []
            if i > 0:
                p.append((lst[i - 1], 0))
            if kd == FWD and prev[k] >= 0:
                p.append(((FWD, prev[k], j), 0 if blocking else pf[prev[k]]))
            if kd == BWD:
                p.append(((BWD, nxt[k], j), 0 if blocking else pb[nxt[k]]) if k in nxt else ((FWD, k, j), 0))
            preds[(kd, k, j)] = p

    def dur(n):
        kd, k, _ = n
        d = Fd[k] if kd == FWD else Bd[k]
        if blocking:
            d += (pf[k] if k in nxt else 0) if kd == FWD else (pb[k] if prev[k] >= 0 else 0)
        return d
    start = {n: 0 for n in preds}
    changed, rounds = True, 0
    while changed:
        changed = False
        rounds += 1
        assert rounds < 20 * len(preds) + 10, "cycle in the task graph"
        for n, ps in preds.items():
            val = max([start[q] + dur(q) + lat for q, lat in ps], default=0)
            if val != start[n]:
                start[n] = val
                changed = True
    return {n: start[n] + dur(n) for n in preds}, start


def random_schedule(rng, pp, S, m):
    """Stages on random devices, split into pipelines (chains), every pipeline with a random subset
    of the micro-batches; execution order = a random linear extension of the task graph."""
    place = [int(rng.integers(0, pp)) for _ in range(S)]
    prev, heads = [-1] * S, []
    k = 0
    while k < S:
        ln = int(rng.integers(1, S - k + 1))
        heads.append((k, ln))
        for q in range(k + 1, k + ln):
            prev[q] = q - 1
        k += ln
    tasks, deps = [], {}
    for (k0, ln) in heads:
        mbs = [j for j in range(m) if rng.random() < 0.7] or [0]
        for j in mbs:
            for q in range(k0, k0 + ln):
                deps[(FWD, q, j)] = [(FWD, q - 1, j)] if q > k0 else []
                deps[(BWD, q, j)] = [(BWD, q + 1, j)] if q + 1 < k0 + ln else [(FWD, q, j)]
    done, order = set(), []
    todo = list(deps)
    while todo:
        ready = [t for t in todo if all(p in done for p in deps[t])]
        t = ready[int(rng.integers(0, len(ready)))]
        order.append(t); done.add(t); todo.remove(t)
    lists = [[t for t in order if place[t[1]] == d] for d in range(pp)]
    return place, prev, lists


def test_random_schedules_against_the_task_graph(oracle_mod):
    rng = np.random.default_rng(99)
    for trial in range(150):
        pp = int(rng.integers(1, 6))
        S = int(rng.integers(1, 9))
        m = int(rng.integers(1, 5))
        nparts = int(rng.integers(1, 5))
        L = nparts + int(rng.integers(0, 4))
        bnd = [0] + sorted(rng.choice(np.arange(1, L), nparts - 1, replace=False).tolist()) + [L]
        place, prev, lists = random_schedule(rng, pp, S, m)
        part = [int(rng.integers(0, nparts)) for _ in range(S)]
        replicas = int(rng.choice([1, 2, 3]))
        dp = int(rng.choice([1, 2]))
        blocking = int(rng.integers(0, 2))
        fc, bc = rng.integers(0, 40, L).tolist(), rng.integers(0, 60, L).tolist()
        act, grad = (rng.integers(0, 9, L) * 5).tolist(), rng.integers(0, 200, L).tolist()
        costs = mk_costs(fc, bc, act=act, grad=grad)
        g = int(rng.choice([1, 2, 1 << 20]))
        cl = mk_cluster(dp * pp, g=g, alpha=(2, 7), beta=(5, 1), blocking=blocking)
        blk = pack_schedule(pp, list(zip(place, part, prev)), m, nparts, replicas, lists)
        w = with_schedules(mk(costs, cl, [(dp, 1, pp, m, 4, bnd, 0)]), [blk], [0])
        r = oracle_mod.simulate(w, timeline=True)
        assert r["status"][0] == 0, trial
        Fd = [sum(fc[bnd[part[k]]:bnd[part[k] + 1]]) for k in range(S)]
        Bd = [sum(bc[bnd[part[k]]:bnd[part[k] + 1]]) for k in range(S)]
        node = lambda d: (d * dp) // g
        pf, pb = [0] * S, [0] * S
        for k in range(S):
            if prev[k] >= 0:
                q = prev[k]
                cls = 0 if node(place[q]) == node(place[k]) else 1
                t = (2, 7)[cls] + act[bnd[part[q] + 1] - 1] // (5, 1)[cls]
                pf[q], pb[k] = t, t
        end, start = longest_path(S, m, place, prev, lists, Fd, Bd, pf, pb, blocking)
        # the dump: every listed task with its start and end, the others untouched
        assert r["start"].shape == (2, S, m)
        for kd in (FWD, BWD):
            for k in range(S):
                for j in range(m):
                    if (kd, k, j) in end:
                        assert r["end"][kd, k, j] == end[(kd, k, j)] and r["start"][kd, k, j] == start[(kd, k, j)], (trial, kd, k, j)
                    else:
                        assert r["end"][kd, k, j] == -1 and r["start"][kd, k, j] == -1
        n = dp * replicas
        has_next = {prev[q] for q in range(S) if prev[q] >= 0}
        fin, comp, comm, nar = [], [], [], 0
        for d in range(pp):
            G = sum(sum(grad[bnd[part[k]]:bnd[part[k] + 1]]) for k in range(S) if place[k] == d)
            last = max([end[t] for t in lists[d]], default=0)
            ar = 0
            if lists[d] and n > 1 and G > 0:
                cls = 0 if n <= g else 1
                ar = (2, 7)[cls] + (2 * (n - 1) * G) // (n * (5, 1)[cls])
                nar += 1
            fin.append(last + ar)
            assert r["ar_window"][0][d] == (last if ar or (lists[d] and n > 1 and G > 0) else -1)
            assert r["ar_window"][1][d] == (last + ar if ar or (lists[d] and n > 1 and G > 0) else -1)
            comp.append(sum(Fd[k] if kd == FWD else Bd[k] for kd, k, _ in lists[d]))
            sends = sum((pf[k] if kd == FWD else pb[k]) for kd, k, _ in lists[d])
            comm.append(sends + ar)
        assert r["batch_ns"][0] == max(fin), trial
        assert list(r["comp_busy_ns"]) == comp and list(r["comm_busy_ns"]) == comm, trial
        ntask = sum(len(x) for x in lists)
        nsend = sum(1 for lst in lists for kd, k, _ in lst if (k in has_next if kd == FWD else prev[k] >= 0))
        assert r["num_events"][0] == ntask + nsend + nar, trial


def test_serialised_links_against_graph_with_send_nodes(oracle_mod):
    """p2p_blocking = 2 for explicit schedules: the sender goes on, every transfer is a node of its own.
    A link is an ordered pair (sending device, receiving device) and carries one transfer at a time:
    a send starts when its task has ended and the send before it on that link (in the order of the
    sending device's list) has arrived; the consumer waits for the arrival.  Solved by relaxation."""
    rng = np.random.default_rng(414)
    queued = 0
    for trial in range(200):
        pp = int(rng.integers(1, 5))
        S = int(rng.integers(1, 9))
        m = int(rng.integers(1, 5))
        nparts = int(rng.integers(1, 5))
        L = nparts + int(rng.integers(0, 4))
        bnd = [0] + sorted(rng.choice(np.arange(1, L), nparts - 1, replace=False).tolist()) + [L]
        place, prev, lists = random_schedule(rng, pp, S, m)
        part = [int(rng.integers(0, nparts)) for _ in range(S)]
        fc, bc = rng.integers(0, 30, L).tolist(), rng.integers(0, 30, L).tolist()
        act = (rng.integers(0, 40, L) * 5).tolist()              # transfers often longer than the tasks
        costs = mk_costs(fc, bc, act=act)
        g = int(rng.choice([1, 2, 1 << 20]))
        blk = pack_schedule(pp, list(zip(place, part, prev)), m, nparts, 1, lists)
        w = with_schedules(mk(costs, mk_cluster(pp, g=g, alpha=(2, 7), beta=(5, 1), blocking=2), [(1, 1, pp, m, 4, bnd, 0)]), [blk], [0])
        r = oracle_mod.simulate(w, timeline=True)
        assert r["status"][0] == 0, trial
        Fd = [sum(fc[bnd[part[k]]:bnd[part[k] + 1]]) for k in range(S)]
        Bd = [sum(bc[bnd[part[k]]:bnd[part[k] + 1]]) for k in range(S)]
        nxt = {prev[k]: k for k in range(S) if prev[k] >= 0}
        pf, pb = [0] * S, [0] * S
        for k in range(S):
            if prev[k] >= 0:
                q = prev[k]
                cls = 0 if place[q] // g == place[k] // g else 1
                t = (2, 7)[cls] + act[bnd[part[q] + 1] - 1] // (5, 1)[cls]
                pf[q], pb[k] = t, t
        dur = lambda n: Fd[n[1]] if n[0] == FWD else Bd[n[1]]
        # where the transfer after a task goes, and how long it takes (None: the task sends nothing)
        def send_of(n):
            kd, k, _ = n
            if kd == FWD and k in nxt:
                return place[nxt[k]], pf[k]
            if kd == BWD and prev[k] >= 0:
                return place[prev[k]], pb[k]
            return None
        preds = {}                     # node -> [(node before it, time from that node's START to this node's start)]
        for d, lst in enumerate(lists):
            last_on_link = {}
            for i, t in enumerate(lst):
                kd, k, j = t
                p = [(("T",) + lst[i - 1], dur(lst[i - 1]))] if i > 0 else []
                if kd == FWD and prev[k] >= 0:
                    p.append((("S", FWD, prev[k], j), pf[prev[k]]))
                if kd == BWD:
                    p.append((("S", BWD, nxt[k], j), pb[nxt[k]]) if k in nxt else (("T", FWD, k, j), Fd[k]))
                preds[("T",) + t] = p
                sd = send_of(t)
                if sd is not None:
                    q = [(("T",) + t, dur(t))]
                    if sd[0] in last_on_link:
                        before = last_on_link[sd[0]]
                        q.append((("S",) + before, send_of(before)[1]))
                    preds[("S",) + t] = q
                    last_on_link[sd[0]] = t
        start = {n: 0 for n in preds}
        changed, rounds = True, 0
        while changed:
            changed = False
            rounds += 1
            assert rounds < 20 * len(preds) + 10
            for n, ps in preds.items():
                val = max([start[q] + wgt for q, wgt in ps], default=0)
                if val != start[n]:
                    start[n] = val
                    changed = True
        for n, val in start.items():
            if n[0] == "T":
                assert r["start"][n[1], n[2], n[3]] == val, (trial, n)
                assert r["end"][n[1], n[2], n[3]] == val + dur(n[1:]), (trial, n)
        assert r["batch_ns"][0] == max(start[("T",) + t] + dur(t) for lst in lists for t in lst), trial
        for d, lst in enumerate(lists):
            assert r["comm_busy_ns"][d] == sum(send_of(t)[1] for t in lst if send_of(t) is not None)
        w.cluster["p2p_blocking"] = 0
        free = oracle_mod.simulate(w)
        assert r["batch_ns"][0] >= free["batch_ns"][0]
        queued += int(r["batch_ns"][0] > free["batch_ns"][0])
    assert queued > 10                 # the queueing really delays a good number of the cases


def test_bidirectional_lists_run_and_use_both_directions(oracle_mod):
    """Two pipelines in opposite directions: every device list is a merge of the two early-backward
    orders; the run ends, both replicas' gradients are reduced over dp * 2 ranks, and with equal
    stages the two directions take the same time (mirror symmetry)."""
    for pp, m in [(2, 2), (4, 4), (4, 8), (6, 6), (8, 8), (8, 16)]:
        L = pp
        costs = mk_costs([100] * L, [200] * L, act=[50] * L, grad=[1000] * L)
        cl = mk_cluster(pp, g=1 << 20, alpha=(0, 0), beta=(10, 10))
        blk = pack_schedule(pp, bidirectional_stages(pp), m, pp, 2, bidirectional_lists(pp, m))
        one = pack_schedule(pp, chain(pp), m, pp, 1, dapple_lists(pp, m))
        w = with_schedules(mk(costs, cl, [(1, 1, pp, m, 4, None, 0), (1, 1, pp, m, 4, None, 1)]), [blk, one], [0, 1])
        r = oracle_mod.simulate(w)
        assert list(r["status"]) == [0, 0]
        so = r["stage_off"]
        comp = r["comp_busy_ns"][so[0]:so[1]]
        assert (comp == m * 300).all()                              # every device: m forwards and m backwards in all
        ar = 2 * 1 * 2 * 1000 // (2 * 10)                           # two ranks, bytes of the device's two stages
        assert r["num_events"][0] == 2 * m * pp + 2 * m * (pp - 1) + pp
        # mirror symmetry: device d and device pp - 1 - d finish together when m is even
        if m % 2 == 0:
            w2 = with_schedules(mk(costs, cl, [(1, 1, pp, m, 4, None, 0)]), [blk], [0])
            assert oracle_mod.simulate(w2)["batch_ns"][0] == r["batch_ns"][0]
        # never slower than running all micro-batches through one pipeline, all-reduce apart
        assert r["batch_ns"][0] - ar <= r["batch_ns"][1]


def test_invalid_explicit_schedules(oracle_mod):
    pp, m = 2, 2
    costs = mk_costs([10] * 4, [20] * 4, act=[30] * 4)
    cl = mk_cluster(pp)
    good = pack_schedule(pp, chain(pp), m, pp, 1, dapple_lists(pp, m))

    def status(blk, ids=(0,), row=(1, 1, pp, m, 4, None, 0), cluster=cl, n_blocks=None):
        w = with_schedules(mk(costs, cluster, [row]), [blk] if n_blocks is None else [blk] * n_blocks, list(ids))
        return int(oracle_mod.simulate(w)["status"][0])
    assert status(good) == 0
    assert status(good, ids=(1,)) == 1 and status(good, ids=(-1,)) == 1            # no such schedule
    assert status(good, row=(1, 1, pp, 3, 4, None, 0)) == 1                          # m differs
    assert status(good, cluster=mk_cluster(pp, blocking=2)) == 0                     # link queues are modelled
    lists = dapple_lists(pp, m)
    swapped = [lists[0], [lists[1][1], lists[1][0]] + lists[1][2:]]                  # B(1,0) before F(1,0): never ready
    assert status(pack_schedule(pp, chain(pp), m, pp, 1, swapped)) == 1
    dup = [lists[0] + [lists[0][0]], lists[1]]
    assert status(pack_schedule(pp, chain(pp), m, pp, 1, dup)) == 1                  # a task twice
    wrongdev = [lists[1], lists[0]]
    assert status(pack_schedule(pp, chain(pp), m, pp, 1, wrongdev)) == 1             # a task on a device that does not hold its stage
    missing = [lists[0][:1] + lists[0][2:], lists[1]]                                # producer of F(1,1) is not there
    assert status(pack_schedule(pp, chain(pp), m, pp, 1, missing)) == 1
    assert status(pack_schedule(pp, [(0, 0, -1), (1, 1, 0), (1, 1, 0)], m, pp, 1, lists)) == 1    # two stages after one
    assert status(pack_schedule(pp, [(0, 0, -1), (2, 1, 0)], m, pp, 1, lists)) == 1               # device out of range
    assert status(pack_schedule(pp, [(0, 0, -1), (1, 2, 0)], m, pp, 1, lists)) == 1               # part out of range
    assert status(pack_schedule(pp, chain(pp), m, pp, 0, lists)) == 1                             # replicas < 1
    assert status(good[:-1]) == 1                                                                  # block too short
    # no tables at all
    w = mk(costs, cl, [(1, 1, pp, m, 4, None)])
    assert int(oracle_mod.simulate(w)["status"][0]) == 1
    # cyclic wait between two devices
    stages = [(0, 0, -1), (1, 1, 0), (1, 0, -1), (0, 1, 2)]                                        # two pipelines, opposite ways
    cyc = [[(FWD, 3, 0), (FWD, 0, 0), (BWD, 0, 0), (BWD, 3, 0)], [(FWD, 1, 0), (FWD, 2, 0), (BWD, 1, 0), (BWD, 2, 0)]]
    assert status(pack_schedule(pp, stages, 1, pp, 1, cyc), row=(1, 1, pp, 1, 4, None, 0)) == 1
    okl = [[(FWD, 0, 0), (FWD, 3, 0), (BWD, 3, 0), (BWD, 0, 0)], [(FWD, 2, 0), (FWD, 1, 0), (BWD, 1, 0), (BWD, 2, 0)]]
    assert status(pack_schedule(pp, stages, 1, pp, 1, okl), row=(1, 1, pp, 1, 4, None, 0)) == 0


def test_pack_and_unpack_are_inverse():
    from workloads.schedules import unpack_schedule
    rng = np.random.default_rng(3)
    for _ in range(50):
        pp, S, m = int(rng.integers(1, 9)), int(rng.integers(1, 20)), int(rng.integers(1, 9))
        place, prev, lists = random_schedule(rng, pp, S, m)
        stages = [(place[k], int(rng.integers(0, 4)), prev[k]) for k in range(S)]
        blk = pack_schedule(pp, stages, m, 4, 2, lists)
        assert blk.dtype == np.int32
        got = unpack_schedule(blk)
        assert got == (pp, stages, m, 4, 2, lists)


def test_generated_lists_are_complete_and_run_to_their_end(oracle_mod):
    """Every generator lists each of its tasks once, on the device that holds the stage, and the
    oracle runs the schedule to its end for every shape tried."""
    for pp in (1, 2, 3, 4, 5, 8, 13, 16):
        for m in (1, 2, 3, 7, 16):
            cases = [(chain(pp), gpipe_lists(pp, m), 1, pp, set(range(m))), (chain(pp), dapple_lists(pp, m), 1, pp, set(range(m)))]
            if pp % 2 == 0:
                cases.append((bidirectional_stages(pp), bidirectional_lists(pp, m), 2, pp, None))
            for v in (1, 2, 3):
                if m % pp == 0 and pp * v <= 16:
                    cases.append((interleaved_stages(pp, v), interleaved_lists(pp, v, m), 1, pp * v, set(range(m))))
            for stages, lists, replicas, nparts, mbs in cases:
                seen = set()
                for d, lst in enumerate(lists):
                    for t in lst:
                        assert t not in seen and stages[t[1]][0] == d
                        seen.add(t)
                if mbs is not None:
                    assert seen == {(kd, k, j) for kd in (FWD, BWD) for k in range(len(stages)) for j in mbs}
                else:                                   # two pipelines: every micro-batch through exactly one of them
                    for j in range(m):
                        pipes = {k // pp for kd, k, jj in seen if jj == j}
                        assert len(pipes) == 1
                L = max(nparts, 2)
                costs = mk_costs([7] * L, [11] * L, act=[64] * L, grad=[100] * L)
                w = with_schedules(mk(costs, mk_cluster(pp), [(1, 1, pp, m, 4, None, 0)]),
                                   [pack_schedule(pp, stages, m, nparts, replicas, lists)], [0])
                assert int(oracle_mod.simulate(w)["status"][0]) == 0, (pp, m, len(stages))
