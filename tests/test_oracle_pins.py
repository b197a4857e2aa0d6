"""Pins for the CPU oracle: things the paper and the mathematics fix, none of them
computed by the oracle itself.

 * hand-unrolled timelines (tests/golden)            -> schedule orders, p2p edges, origin
 * closed forms (uniform pipeline, GPipe flow shop)   -> recurrence, DP tail
 * explicit task graph + longest path (brute force)   -> every timestamp, both schedules
 * Dapple's in-flight bound                           -> 1F1B order
 * ring all-reduce volume 2(N-1)P/N (Sec. 4.2)        -> collective costs
 * invariants / metamorphic relations                 -> busy accounting, isotonicity
 * facts printed in the paper (Sec. 5.4, Sec. 6)       -> event counts, grid size
"""
import itertools
import os

import numpy as np
import pytest

from helpers import mk, mk_cluster, mk_costs
from workloads import enumerate_triples, make_workload, subset

GOLD = os.path.join(os.path.dirname(__file__), "golden")
INT64_MAX = np.iinfo(np.int64).max


# ----------------------------------------------------------------------------- helpers

def one(oracle, costs, cluster, row, timeline=False):
    r = oracle.simulate(mk(costs, cluster, [row]), timeline=timeline)
    return r


def device_order(sched, pp, m, s):
    """Per-device task order, written from the schedules' definitions (GPipe: all forwards
    then all backwards; Dapple: at most pp - s micro-batches in flight on stage s)."""
    if sched == 0:
        return [("F", j) for j in range(m)] + [("B", j) for j in range(m)]
    out, f, b = [], 0, 0
    limit = pp - s
    while b < m:
        if f < m and f - b < limit:
            out.append(("F", f)); f += 1
        else:
            out.append(("B", b)); b += 1
    return out


def longest_path(sched, pp, m, F, B, pf, pb):
    """start/end of every task from the explicit dependency graph, by relaxation to a fixpoint
    (no event queue, no levels).  pf[s]: latency s -> s+1, pb[s]: latency s -> s-1."""
    preds = {}
    for s in range(pp):
        order = device_order(sched, pp, m, s)
        for i, (k, j) in enumerate(order):
            p = []
            if i > 0:
                pk, pj = order[i - 1]
                p.append(((pk, s, pj), 0))
            if k == "F" and s > 0:
                p.append((("F", s - 1, j), pf[s - 1]))
            if k == "B" and s < pp - 1:
                p.append((("B", s + 1, j), pb[s + 1]))
            if k == "B" and s == pp - 1:
                p.append((("F", s, j), 0))
            preds[(k, s, j)] = p
    dur = lambda n: F[n[1]] if n[0] == "F" else B[n[1]]
    start = {n: 0 for n in preds}
    changed = True
    rounds = 0
    while changed:
        changed = False
        rounds += 1
        assert rounds < 10 * len(preds) + 10, "cycle in the task graph"
        for n, ps in preds.items():
            v = 0
            for (q, lat) in ps:
                v = max(v, start[q] + dur(q) + lat)
            if v != start[n]:
                start[n] = v
                changed = True
    end = {n: start[n] + dur(n) for n in preds}
    return start, end


# ----------------------------------------------------------------------------- golden

def _read_golden_pipeline():
    rows = []
    with open(os.path.join(GOLD, "pipeline_pp2_m4.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            sc, k, s, j, a, b, c = line.split()
            rows.append((sc, k, int(s), int(j), int(a), int(b), int(c)))
    return rows


@pytest.mark.parametrize("f,b,alpha,act", [
    (1_000_000, 2_025_000, 5000, 4 << 20),   # the Tiny workload's numbers
    (7, 3, 0, 0), (5, 11, 1, 200 * 13), (100, 100, 1000, 0), (0, 9, 4, 0),
])
def test_golden_pp2_m4_timeline(oracle_mod, f, b, alpha, act):
    rows = _read_golden_pipeline()
    costs = mk_costs([f] * 4, [b] * 4, act=[act] * 4)
    cl = mk_cluster(2, alpha=(alpha, 77777), beta=(200, 1))
    F, B, c = 2 * f, 2 * b, alpha + act // 200
    for sc_name, sc in (("1f1b", 1), ("gpipe", 0)):
        r = one(oracle_mod, costs, cl, (1, 1, 2, 4, sc, [0, 2, 4]), timeline=True)
        assert r["status"][0] == 0
        n = 0
        for (name, k, s, j, a, bb, cc) in rows:
            if name != sc_name:
                continue
            n += 1
            kd = 0 if k == "F" else 1
            st = a * F + bb * B + cc * c
            assert r["start"][kd, s, j] == st, (name, k, s, j)
            assert r["end"][kd, s, j] == st + (F if kd == 0 else B)
        assert n == 16
        want = 5 * (F + B) + (4 if sc == 1 else 2) * c
        assert r["batch_ns"][0] == want
        assert list(r["comp_busy_ns"]) == [4 * (F + B)] * 2
        assert list(r["comm_busy_ns"]) == [4 * c] * 2
        assert r["num_events"][0] == 16 + 8


def test_golden_tiny_numbers(oracle_mod):
    costs = mk_costs([1_000_000] * 4, [2_025_000] * 4, act=[4 << 20] * 4)
    w = mk(costs, mk_cluster(2), [(1, 1, 2, 4, 1, [0, 2, 4]), (1, 1, 2, 4, 0, [0, 2, 4])])
    r = oracle_mod.simulate(w)
    assert list(r["batch_ns"]) == [30_353_884, 30_301_942]
    assert np.allclose(r["util"][:2], 24_200_000 / 30_353_884, rtol=1e-15)


def test_golden_bucketed_allreduce(oracle_mod):
    n = 0
    with open(os.path.join(GOLD, "bucketed_allreduce.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, dp, g0, g1, g2, batch, comm, nar, ar0, ar1 = line.split()
            dp = int(dp)
            costs = mk_costs([10, 10, 10], [50, 300, 500], grad=[int(g0), int(g1), int(g2)])
            cl = mk_cluster(dp, g=8, alpha=(100, 100), beta=(10, 10), bucket=1000)
            r = one(oracle_mod, costs, cl, (dp, 1, 1, 1, 0, None), timeline=True)
            assert r["batch_ns"][0] == int(batch), name
            assert list(r["ar_window"][:, 0]) == [int(ar0), int(ar1)], name
            assert r["comm_busy_ns"][0] == int(comm), name
            assert r["num_events"][0] == 2 + int(nar), name
            assert r["comp_busy_ns"][0] == 880
            n += 1
    assert n == 5


# ----------------------------------------------------------------------------- closed forms

@pytest.mark.parametrize("sched", [0, 1])
def test_uniform_pipeline_closed_form(oracle_mod, sched):
    """Equal stages, zero p2p: batch = (m + pp - 1)(tF + tB) + trailing all-reduce."""
    rng = np.random.default_rng(5)
    rows, want = [], []
    L = 24
    f, b, g = 1234, 2777, 4096
    for pp in (1, 2, 3, 4, 6, 8, 12, 24):
        for m in (1, 2, 3, 7, 16, 33):
            for dp in (1, 2, 16):
                rows.append((dp, 1, pp, m, sched, None, ))
    costs = mk_costs([f] * L, [b] * L, act=[0] * L, grad=[g] * L)
    for (dp, tp, pp, m, sc, _) in rows:
        N = dp * pp
        cl = mk_cluster(N, alpha=(0, 0), beta=(200, 25))
        r = one(oracle_mod, costs, cl, (dp, 1, pp, m, sc, None))
        lay = L // pp
        n = dp
        beta = 200 if n <= 8 else 25
        ar = 0 if n == 1 else (2 * (n - 1) * g * lay) // (n * beta)
        assert r["batch_ns"][0] == (m + pp - 1) * lay * (f + b) + ar, (dp, pp, m)


def _stage_sums(x, bnd):
    return [sum(x[bnd[s]:bnd[s + 1]]) for s in range(len(bnd) - 1)]


def test_gpipe_flow_shop_closed_form(oracle_mod):
    """GPipe with identical micro-batches is a permutation flow shop with identical jobs:
    forward phase ends at sum F + sum pf + (m-1) max F; the backward wave then reaches stage s
    at T_fwd + sum_{i>=s} B_i + sum_{i>s} pb_i + (m-1) max_{i>=s} B_i."""
    rng = np.random.default_rng(11)
    L = 12
    for trial in range(300):
        pp = int(rng.integers(1, 7))
        m = int(rng.integers(1, 9))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 1000, L).tolist()
        bc = rng.integers(0, 2000, L).tolist()
        act = (rng.integers(0, 50, L) * 200).tolist()
        grad = rng.integers(1, 5000, L).tolist()
        dp = int(rng.choice([1, 2, 4]))
        alpha = int(rng.integers(0, 300))
        costs = mk_costs(fc, bc, act=act, grad=grad)
        cl = mk_cluster(dp * pp, g=1 << 20, alpha=(alpha, 0), beta=(200, 1))
        r = one(oracle_mod, costs, cl, (dp, 1, pp, m, 0, bnd))
        F, B, G = _stage_sums(fc, bnd), _stage_sums(bc, bnd), _stage_sums(grad, bnd)
        pf = [alpha + act[bnd[s + 1] - 1] // 200 for s in range(pp - 1)]
        t_fwd = sum(F) + sum(pf) + (m - 1) * max(F)
        batch = 0
        for s in range(pp):
            e = t_fwd + sum(B[s:]) + sum(pf[s:]) + (m - 1) * max(B[s:])
            ar = 0 if dp == 1 else alpha + (2 * (dp - 1) * G[s]) // (dp * 200)
            batch = max(batch, e + ar)
        assert r["batch_ns"][0] == batch, (trial, pp, m, bnd)


@pytest.mark.parametrize("blocking", [0, 1, 2])
def test_gpipe_flow_shop_every_task(oracle_mod, blocking):
    """The same flow shop, task by task: end F(s, j) = sum_{i<=s} (F_i + pf_i) + j max_{i<=s} F_i and
    end B(s, j) = end F(pp-1, m-1) + sum_{i>=s} (B_i + pb_i) + j max_{i>=s} B_i.  A sender that is
    occupied by its send (p2p_blocking = 1) has the send in its task and the edge costs nothing; a link
    that carries one transfer at a time (p2p_blocking = 2) is one more machine between its two stages,
    so its transfer time is among the maxima."""
    rng = np.random.default_rng(12)
    L = 16
    for trial in range(200):
        pp = int(rng.integers(1, 12))
        m = int(rng.integers(1, 10))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 1000, L).tolist()
        bc = rng.integers(0, 2000, L).tolist()
        act = (rng.integers(0, 400, L) * 200).tolist()                          # transfers as long as stage-tasks
        alpha = int(rng.integers(0, 300))
        costs = mk_costs(fc, bc, act=act)
        cl = mk_cluster(pp, g=1 << 20, alpha=(alpha, 0), beta=(200, 1), blocking=blocking)
        r = one(oracle_mod, costs, cl, (1, 1, pp, m, 0, bnd), timeline=True)
        F, B = _stage_sums(fc, bnd), _stage_sums(bc, bnd)
        edge = [alpha + act[bnd[s + 1] - 1] // 200 for s in range(pp - 1)]      # between s and s + 1
        if blocking == 1:
            F = [F[s] + (edge[s] if s + 1 < pp else 0) for s in range(pp)]
            B = [B[s] + (edge[s - 1] if s > 0 else 0) for s in range(pp)]
            edge = [0] * (pp - 1)
        queue = blocking == 2
        endF = lambda s, j: sum(F[:s + 1]) + sum(edge[:s]) + j * max(F[:s + 1] + (edge[:s] if queue else []))
        R = endF(pp - 1, m - 1)
        endB = lambda s, j: R + sum(B[s:]) + sum(edge[s:]) + j * max(B[s:] + (edge[s:] if queue else []))
        for s in range(pp):
            for j in range(m):
                assert r["end"][0, s, j] == endF(s, j), (trial, "F", s, j)
                assert r["end"][1, s, j] == endB(s, j), (trial, "B", s, j)


@pytest.mark.parametrize("blocking", [0, 1, 2])
@pytest.mark.parametrize("sched", [1, 2])
def test_early_backward_warm_up_is_a_flow_shop(oracle_mod, sched, blocking):
    """The forwards that a stage of the early-backward schedule runs in front of its first backward,
    F(s, j) with j <= min(pp - 1 - s, m - 1), depend only on forwards of the same set, so they pass the
    stages as identical jobs pass the machines of a flow shop:
    end F(s, j) = sum_{i<=s} (F_i + pf_i) + j max_{i<=s} F_i, whatever the backwards behind them do
    (with one transfer per link at a time, p2p_blocking = 2, the links in front of s join the maximum)."""
    rng = np.random.default_rng(21)
    L = 16
    for trial in range(200):
        pp = int(rng.integers(1, 12))
        m = int(rng.integers(1, 14))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 1000, L).tolist()
        bc = rng.integers(0, 2000, L).tolist()
        act = (rng.integers(0, 400, L) * 200).tolist()
        alpha = int(rng.integers(0, 300))
        costs = mk_costs(fc, bc, act=act)
        cl = mk_cluster(pp, g=1 << 20, alpha=(alpha, 0), beta=(200, 1), blocking=blocking)
        r = one(oracle_mod, costs, cl, (1, 1, pp, m, sched, bnd), timeline=True)
        F = _stage_sums(fc, bnd)
        edge = [alpha + act[bnd[s + 1] - 1] // 200 for s in range(pp - 1)]      # between s and s + 1
        if blocking == 1:
            F = [F[s] + (edge[s] if s + 1 < pp else 0) for s in range(pp)]
            edge = [0] * (pp - 1)
        for s in range(pp):
            for j in range(min(pp - 1 - s, m - 1) + 1):
                top = max(F[:s + 1] + (edge[:s] if blocking == 2 else []))
                assert r["end"][0, s, j] == sum(F[:s + 1]) + sum(edge[:s]) + j * top, (trial, s, j)


@pytest.mark.parametrize("sched", [0, 1])
def test_degenerate_cases(oracle_mod, sched):
    L = 6
    fc, bc = [3, 5, 7, 11, 13, 17], [19, 23, 29, 31, 37, 41]
    act = [200 * k for k in (1, 2, 3, 4, 5, 6)]
    costs = mk_costs(fc, bc, act=act, grad=[1000] * L)
    # no pipeline: one sequential stage (Sec. 4.3), m (F + B) + all-reduce
    for m in (1, 5):
        cl = mk_cluster(4, alpha=(10, 10), beta=(200, 200))
        r = one(oracle_mod, costs, cl, (4, 1, 1, m, sched, None))
        ar = 10 + (2 * 3 * 6000) // (4 * 200)
        assert r["batch_ns"][0] == m * (sum(fc) + sum(bc)) + ar
        assert r["num_events"][0] == 2 * m + 1
    # one micro-batch: a single round trip through the stages
    bnd = [0, 1, 3, 6]
    cl = mk_cluster(3, alpha=(10, 10), beta=(200, 200))
    r = one(oracle_mod, costs, cl, (1, 1, 3, 1, sched, bnd))
    p = [10 + act[0] // 200, 10 + act[2] // 200]
    assert r["batch_ns"][0] == sum(fc) + sum(bc) + 2 * sum(p)


# ----------------------------------------------------------------------------- brute force

def test_brute_force_longest_path_all_timestamps(oracle_mod):
    rng = np.random.default_rng(7)
    L = 6
    checked = 0
    for trial in range(400):
        pp = int(rng.integers(1, 5))
        m = int(rng.integers(1, 7))
        sched = int(rng.integers(0, 2))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        hi = int(rng.choice([2, 10, 1000]))
        fc = rng.integers(0, hi, L).tolist()
        bc = rng.integers(0, hi, L).tolist()
        fa = rng.integers(0, hi, L).tolist()
        ba = rng.integers(0, hi, L).tolist()
        tp = int(rng.choice([1, 2]))
        act = (rng.integers(0, 4, L) * 5).tolist()
        alpha = int(rng.integers(0, hi))
        costs = mk_costs(fc, bc, fa=fa, ba=ba, act=act, tps=(tp,))
        cl = mk_cluster(tp * pp, g=1 << 20, alpha=(alpha, 0), beta=(5, 1))
        r = one(oracle_mod, costs, cl, (1, tp, pp, m, sched, bnd), timeline=True)
        assert r["status"][0] == 0
        comm = (lambda x: x) if tp > 1 else (lambda x: [0] * L)
        F = [a + b for a, b in zip(_stage_sums(fc, bnd), _stage_sums(comm(fa), bnd))]
        B = [a + b for a, b in zip(_stage_sums(bc, bnd), _stage_sums(comm(ba), bnd))]
        pf = [alpha + act[bnd[s + 1] - 1] // 5 for s in range(pp - 1)] + [0]
        pb = [0] + [alpha + act[bnd[s] - 1] // 5 for s in range(1, pp)]
        start, end = longest_path(sched, pp, m, F, B, pf, pb)
        for (k, s, j), v in start.items():
            kd = 0 if k == "F" else 1
            assert r["start"][kd, s, j] == v, (trial, k, s, j)
            assert r["end"][kd, s, j] == end[(k, s, j)]
        assert r["batch_ns"][0] == max(end.values())
        # busy = sum of event durations on the device's list
        for s in range(pp):
            assert r["comp_busy_ns"][s] == m * (sum(fc[bnd[s]:bnd[s + 1]]) + sum(bc[bnd[s]:bnd[s + 1]]))
            cm = m * (F[s] + B[s]) - r["comp_busy_ns"][s]
            cm += m * (pf[s] if s < pp - 1 else 0) + m * (pb[s] if s > 0 else 0)
            assert r["comm_busy_ns"][s] == cm
        checked += 1
    assert checked == 400


def test_blocking_p2p_against_task_graph(oracle_mod):
    """p2p_blocking = 1: the send occupies the sender, so it is the tail of the stage-task and
    the edge to the neighbour has no latency left.  Same task graph, durations F + pf / B + pb."""
    rng = np.random.default_rng(21)
    L = 6
    for trial in range(300):
        pp = int(rng.integers(1, 5))
        m = int(rng.integers(1, 7))
        sched = int(rng.integers(0, 2))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 50, L).tolist()
        bc = rng.integers(0, 50, L).tolist()
        act = (rng.integers(0, 9, L) * 5).tolist()
        dp = int(rng.choice([1, 2]))
        costs = mk_costs(fc, bc, act=act, grad=[100] * L)
        cl = mk_cluster(dp * pp, g=1 << 20, alpha=(2, 0), beta=(5, 1), blocking=1)
        r = one(oracle_mod, costs, cl, (dp, 1, pp, m, sched, bnd), timeline=True)
        pf = [2 + act[bnd[s + 1] - 1] // 5 for s in range(pp - 1)] + [0]
        pb = [0] + [2 + act[bnd[s] - 1] // 5 for s in range(1, pp)]
        F = [a + b for a, b in zip(_stage_sums(fc, bnd), pf)]
        B = [a + b for a, b in zip(_stage_sums(bc, bnd), pb)]
        start, end = longest_path(sched, pp, m, F, B, [0] * pp, [0] * pp)
        for (k, s, j), v in start.items():
            kd = 0 if k == "F" else 1
            assert r["start"][kd, s, j] == v, (trial, k, s, j)
            assert r["end"][kd, s, j] == end[(k, s, j)]
        G = [100 * (bnd[s + 1] - bnd[s]) for s in range(pp)]
        ar = [0 if dp == 1 else 2 + (2 * (dp - 1) * g) // (dp * 5) for g in G]
        assert r["batch_ns"][0] == max(end[("B", s, m - 1)] + ar[s] for s in range(pp))
        for s in range(pp):
            assert r["comm_busy_ns"][s] == m * (pf[s] + pb[s]) + ar[s]
    # against the latency reading: blocking can only delay
    w = make_workload("gpt24")
    from workloads import Workload
    cl = dict(w.cluster); cl["p2p_blocking"] = 1
    a = oracle_mod.simulate(w)
    b = oracle_mod.simulate(Workload("x", w.costs, cl, w.cand))
    assert np.all(b["batch_ns"] >= a["batch_ns"]) and np.any(b["batch_ns"] > a["batch_ns"])
    assert np.array_equal(a["comm_busy_ns"], b["comm_busy_ns"])


def test_serialised_links_against_graph_with_send_nodes(oracle_mod):
    """p2p_blocking = 2: sends do not occupy the device but queue on their link.  Graph: every task
    and every send is a node; a send starts after its task has ended and after the previous send on
    the same link has arrived; the consumer starts after the send has arrived.  Solved by relaxation."""
    rng = np.random.default_rng(33)
    L = 6
    slower = 0
    for trial in range(300):
        pp = int(rng.integers(1, 5))
        m = int(rng.integers(1, 7))
        sched = int(rng.integers(0, 3))
        cuts = sorted(rng.choice(np.arange(1, L), size=pp - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 30, L).tolist()
        bc = rng.integers(0, 30, L).tolist()
        act = (rng.integers(0, 40, L) * 5).tolist()          # sends often longer than the tasks
        costs = mk_costs(fc, bc, act=act)
        cl = mk_cluster(pp, g=1 << 20, alpha=(2, 0), beta=(5, 1), blocking=2)
        r = one(oracle_mod, costs, cl, (1, 1, pp, m, sched, bnd), timeline=True)
        pf = [2 + act[bnd[s + 1] - 1] // 5 for s in range(pp - 1)] + [0]
        pb = [0] + [2 + act[bnd[s] - 1] // 5 for s in range(1, pp)]
        F, B = _stage_sums(fc, bnd), _stage_sums(bc, bnd)
        dur = lambda k, s: F[s] if k == "F" else B[s]
        # nodes ("T", k, s, j) and ("S", k, s, j); preds as (node, weight added to the node's START)
        preds = {}
        for s in range(pp):
            order = device_order(1 if sched else 0, pp, m, s)
            for i, (k, j) in enumerate(order):
                p = []
                if i > 0:
                    pk, pj = order[i - 1]
                    p.append((("T", pk, s, pj), dur(pk, s)))
                if k == "F" and s > 0:
                    p.append((("S", "F", s - 1, j), pf[s - 1]))
                if k == "B" and s < pp - 1:
                    p.append((("S", "B", s + 1, j), pb[s + 1]))
                if k == "B" and s == pp - 1:
                    p.append((("T", "F", s, j), F[s]))
                preds[("T", k, s, j)] = p
            for j in range(m):
                if s < pp - 1:
                    p = [(("T", "F", s, j), F[s])]
                    if j > 0:
                        p.append((("S", "F", s, j - 1), pf[s]))
                    preds[("S", "F", s, j)] = p
                if s > 0:
                    p = [(("T", "B", s, j), B[s])]
                    if j > 0:
                        p.append((("S", "B", s, j - 1), pb[s]))
                    preds[("S", "B", s, j)] = p
        start = {n: 0 for n in preds}
        changed, rounds = True, 0
        while changed:
            changed = False
            rounds += 1
            assert rounds < 10 * len(preds) + 10
            for n, ps in preds.items():
                v = max([start[q] + wgt for q, wgt in ps], default=0)
                if v != start[n]:
                    start[n] = v
                    changed = True
        for n, v in start.items():
            if n[0] != "T":
                continue
            kd = 0 if n[1] == "F" else 1
            assert r["start"][kd, n[2], n[3]] == v, (trial, n)
            assert r["end"][kd, n[2], n[3]] == v + dur(n[1], n[2])
        assert r["batch_ns"][0] == max(start[("T", "B", s, m - 1)] + B[s] for s in range(pp))
        for s in range(pp):
            assert r["comm_busy_ns"][s] == m * (pf[s] + pb[s])
        free = one(oracle_mod, costs, mk_cluster(pp, g=1 << 20, alpha=(2, 0), beta=(5, 1)), (1, 1, pp, m, sched, bnd))
        assert r["batch_ns"][0] >= free["batch_ns"][0]
        slower += int(r["batch_ns"][0] > free["batch_ns"][0])
    assert slower > 10            # the queueing really bites in a good number of the cases
    # sends shorter than every task never queue: same result as the latency reading
    costs = mk_costs([50] * 6, [70] * 6, act=[5] * 6)
    for sched in (0, 1):
        a = one(oracle_mod, costs, mk_cluster(3, g=1 << 20, alpha=(2, 0), beta=(5, 1)), (1, 1, 3, 5, sched, None))
        b = one(oracle_mod, costs, mk_cluster(3, g=1 << 20, alpha=(2, 0), beta=(5, 1), blocking=2), (1, 1, 3, 5, sched, None))
        assert a["batch_ns"][0] == b["batch_ns"][0]


def test_exhaustive_partitions_small(oracle_mod):
    """Every partition of L = 5 layers, both schedules, m = 1..4, against the task graph."""
    L = 5
    fc, bc = [4, 0, 9, 2, 6], [1, 8, 0, 5, 3]
    act = [10, 0, 20, 5, 15]
    costs = mk_costs(fc, bc, act=act)
    for pp in range(1, L + 1):
        for cuts in itertools.combinations(range(1, L), pp - 1):
            bnd = [0] + list(cuts) + [L]
            for sched in (0, 1):
                for m in range(1, 5):
                    cl = mk_cluster(pp, alpha=(3, 3), beta=(5, 5))
                    r = one(oracle_mod, costs, cl, (1, 1, pp, m, sched, bnd))
                    F, B = _stage_sums(fc, bnd), _stage_sums(bc, bnd)
                    pf = [3 + act[bnd[s + 1] - 1] // 5 for s in range(pp - 1)] + [0]
                    pb = [0] + [3 + act[bnd[s] - 1] // 5 for s in range(1, pp)]
                    _, end = longest_path(sched, pp, m, F, B, pf, pb)
                    assert r["batch_ns"][0] == max(end.values()), (bnd, sched, m)


# ----------------------------------------------------------------------------- schedule shape

@pytest.mark.parametrize("pp,m", [(4, 8), (4, 2), (6, 6), (3, 1), (8, 20)])
def test_inflight_bound_of_early_backward(oracle_mod, pp, m):
    """Dapple's early backward keeps at most pp - s micro-batches alive on stage s (forward
    started, backward not finished); GPipe keeps all m."""
    L = pp
    costs = mk_costs([5] * L, [9] * L, act=[0] * L)
    cl = mk_cluster(pp, alpha=(1, 1))
    for sched in (0, 1):
        r = one(oracle_mod, costs, cl, (1, 1, pp, m, sched, None), timeline=True)
        for s in range(pp):
            ev = [(int(t), 1) for t in r["start"][0, s]] + [(int(t), -1) for t in r["end"][1, s]]
            ev.sort(key=lambda x: (x[0], x[1]))
            live = peak = 0
            for _, d in ev:
                live += d
                peak = max(peak, live)
            assert peak == (m if sched == 0 else min(pp - s, m)), (sched, s)
        # every device runs one task at a time, in one order
        for s in range(pp):
            iv = sorted([(int(r["start"][k, s, j]), int(r["end"][k, s, j])) for k in (0, 1) for j in range(m)])
            for a, b in zip(iv, iv[1:]):
                assert a[1] <= b[0]


# ----------------------------------------------------------------------------- collectives

def _ar_via_oracle(oracle, n, P, g=8, alpha=(5000, 10000), beta=(200, 25)):
    costs = mk_costs([0], [0], grad=[P])
    r = one(oracle, costs, mk_cluster(n, g=g, alpha=alpha, beta=beta), (n, 1, 1, 1, 0, None))
    return int(r["batch_ns"][0])


def test_ring_allreduce_volume(oracle_mod):
    P = 3_600_000_000
    assert _ar_via_oracle(oracle_mod, 1, P) == 0                      # no partner, no event
    assert _ar_via_oracle(oracle_mod, 2, P) == 5000 + P // 200        # 2(N-1)/N = 1
    assert _ar_via_oracle(oracle_mod, 8, P) == 5000 + (14 * P) // (8 * 200)
    assert _ar_via_oracle(oracle_mod, 16, P) == 10000 + (30 * P) // (16 * 25)   # > 8 ranks: inter-node
    prev = 0
    for n in (2, 3, 4, 5, 6, 7, 8):
        t = _ar_via_oracle(oracle_mod, n, P)
        assert t > prev
        prev = t
    # volume tends to 2P for many ranks
    t = _ar_via_oracle(oracle_mod, 1 << 20, P, g=1 << 30, alpha=(0, 0))
    assert abs(t - 2 * P // 200) <= 2 * P // 200 // (1 << 19)
    # extrapolation rule of Sec. 4.2: time beyond 8 ranks follows the volume ratio [2(N-1)/N] / [2*7/8]
    for n in (16, 64, 1024):
        t8 = _ar_via_oracle(oracle_mod, 8, P, g=1 << 30, alpha=(0, 0))
        tn = _ar_via_oracle(oracle_mod, n, P, g=1 << 30, alpha=(0, 0))
        assert abs(tn - t8 * (8 * (n - 1)) / (7 * n)) <= 2


def test_p2p_link_class_and_alltoall(oracle_mod):
    # 2 devices in one node: intra-node p2p (Tiny: 5000 + 4 MiB / 200 B/ns = 25 971)
    costs = mk_costs([0, 0], [0, 0], act=[4 << 20, 0])
    r = one(oracle_mod, costs, mk_cluster(2), (1, 1, 2, 1, 0, None))
    assert r["batch_ns"][0] == 2 * 25_971
    # tp*dp = 8 = node size: every boundary crosses nodes
    r = one(oracle_mod, mk_costs([0, 0], [0, 0], act=[4 << 20, 0], tps=(8,)), mk_cluster(16), (1, 8, 2, 1, 0, None))
    assert r["batch_ns"][0] == 2 * (10_000 + (4 << 20) // 25)
    # tp*dp = 4, pp = 4: stages 0,1 share node 0, stages 2,3 share node 1; boundary 1|2 is inter-node
    costs = mk_costs([0] * 4, [0] * 4, act=[200, 400, 800, 0], tps=(4,))
    r = one(oracle_mod, costs, mk_cluster(16), (1, 4, 4, 1, 0, None))
    want = 2 * ((5000 + 1) + (10_000 + 400 // 25) + (5000 + 4))
    assert r["batch_ns"][0] == want
    assert list(r["comm_busy_ns"]) == [5001, 5001 + 10016, 10016 + 5004, 5004]
    # the data-parallel replicas sit between the stages in rank order (tp fastest, then dp, then pp):
    # tp = 2, dp = 2 puts 4 ranks on a stage, so again stages 0,1 | 2,3 and one inter-node boundary;
    # with dp = 1 (2 ranks per stage) all four stages share a node
    costs = mk_costs([0] * 4, [0] * 4, act=[200, 400, 800, 0], tps=(2,), grad=[0] * 4)
    r = one(oracle_mod, costs, mk_cluster(16), (2, 2, 4, 1, 0, None))
    assert r["batch_ns"][0] == 2 * ((5000 + 1) + (10_000 + 400 // 25) + (5000 + 4))
    r = one(oracle_mod, costs, mk_cluster(8), (1, 2, 4, 1, 0, None))
    assert r["batch_ns"][0] == 2 * ((5000 + 1) + (5000 + 2) + (5000 + 4))
    # all-to-all: (n-1)/n of the bytes leave each rank
    costs = mk_costs([7], [9], a2a=[8000], grad=[0])
    for n, want in ((1, 0), (2, 5000 + 4000 // 200), (8, 5000 + (7 * 8000) // (8 * 200)), (16, 10_000 + (15 * 8000) // (16 * 25))):
        r = one(oracle_mod, costs, mk_cluster(n), (n, 1, 1, 3, 0, None))
        assert r["batch_ns"][0] == 3 * (16 + 2 * want)
        assert r["comm_busy_ns"][0] == 6 * want
        assert r["comp_busy_ns"][0] == 48


def test_model_parallel_mapping(oracle_mod):
    """MP = 1: a layer is one computation event; MP > 1: computation + all-reduce (Sec. 4.3)."""
    fc, bc, fa, ba = [[5, 6], [3, 4]], [[7, 8], [5, 6]], [[100, 100], [11, 13]], [[100, 100], [17, 19]]
    costs = mk_costs(fc, bc, fa=fa, ba=ba, tps=(1, 2))
    r = one(oracle_mod, costs, mk_cluster(1), (1, 1, 1, 2, 0, None))
    assert r["batch_ns"][0] == 2 * 26 and r["comm_busy_ns"][0] == 0      # table's comm column ignored for tp = 1
    r = one(oracle_mod, costs, mk_cluster(2), (1, 2, 1, 2, 0, None))
    assert r["batch_ns"][0] == 2 * (18 + 60)
    assert r["comp_busy_ns"][0] == 36 and r["comm_busy_ns"][0] == 120


# ----------------------------------------------------------------------------- invariants / metamorphic

def _random_rows(rng, w, n):
    return rng.choice(w.C, size=n, replace=False)


@pytest.mark.parametrize("name", ["gpt24", "gpt48", "gpt96", "hetero64"])
def test_invariants_on_workloads(oracle_mod, name):
    kw = {"C": 20000} if name == "hetero64" else {}
    w = make_workload(name, **kw)
    rng = np.random.default_rng(3)
    idx = np.sort(_random_rows(rng, w, min(w.C, 300)))
    ws = subset(w, idx)
    r = oracle_mod.simulate(ws, nthreads=4)
    assert (r["status"] == 0).all()
    off = r["stage_off"]
    for i in range(ws.C):
        pp, m = int(ws.cand["pp"][i]), int(ws.cand["m"][i])
        cb = r["comp_busy_ns"][off[i]:off[i + 1]]
        assert len(cb) == pp
        # a device is busy computing one task at a time, so batch >= its compute busy time
        assert r["batch_ns"][i] >= cb.max()
        u = r["util"][off[i]:off[i + 1]]
        assert np.all(u == cb.astype(np.float64) / float(r["batch_ns"][i]))
        assert r["num_events"][i] >= 2 * m * pp + 2 * m * (pp - 1)


def test_metamorphic(oracle_mod):
    w = make_workload("gpt24")
    rng = np.random.default_rng(9)
    idx = np.sort(rng.choice(w.C, 120, replace=False))
    ws = subset(w, idx)
    base = oracle_mod.simulate(ws)
    # homogeneity: scale every duration and alpha by k, beta stays -> bytes/beta must scale too: use bytes*k
    k = 3
    c2 = {key: (v * k if isinstance(v, np.ndarray) and key.endswith(("_ns", "_bytes")) else v) for key, v in w.costs.items()}
    cl2 = dict(w.cluster); cl2["alpha_ns"] = tuple(a * k for a in w.cluster["alpha_ns"])
    from workloads import Workload
    r2 = oracle_mod.simulate(Workload("x", c2, cl2, ws.cand))
    # floor(k*x / b) >= k*floor(x/b); equality needs divisibility, so only bound it
    assert np.all(r2["batch_ns"] >= k * base["batch_ns"])
    assert np.all(r2["batch_ns"] <= k * base["batch_ns"] + k * 4 * 64 * 600)
    assert np.array_equal(r2["comp_busy_ns"], k * base["comp_busy_ns"])
    # isotone: raising one layer's forward time never shortens any candidate
    c3 = {key: (v.copy() if isinstance(v, np.ndarray) else v) for key, v in w.costs.items()}
    c3["fwd_comp_ns"][:, 5] += 12345
    r3 = oracle_mod.simulate(Workload("x", c3, w.cluster, ws.cand))
    assert np.all(r3["batch_ns"] >= base["batch_ns"])
    assert np.any(r3["batch_ns"] > base["batch_ns"])
    # a huge bucket is one all-reduce after the last backward == the paper's trailing event
    cl4 = dict(w.cluster); cl4["dp_bucket_bytes"] = 1 << 60
    r4 = oracle_mod.simulate(Workload("x", w.costs, cl4, ws.cand))
    for key in ("batch_ns", "comp_busy_ns", "comm_busy_ns", "num_events"):
        assert np.array_equal(r4[key], base[key]), key
    # small buckets overlap with the backward: never later than trailing when alpha = 0 ... but
    # each bucket pays alpha; with alpha = 0 and beta | sizes the bucketed finish cannot be later
    cl5 = dict(w.cluster); cl5["alpha_ns"] = (0, 0); cl5["dp_bucket_bytes"] = 0
    cl6 = dict(cl5); cl6["dp_bucket_bytes"] = 25 << 20
    r5 = oracle_mod.simulate(Workload("x", w.costs, cl5, ws.cand))
    r6 = oracle_mod.simulate(Workload("x", w.costs, cl6, ws.cand))
    assert np.all(r6["batch_ns"] <= r5["batch_ns"])
    assert np.any(r6["batch_ns"] < r5["batch_ns"])


def test_dp_changes_only_the_tail(oracle_mod):
    L = 8
    rng = np.random.default_rng(2)
    costs = mk_costs(rng.integers(1, 999, L).tolist(), rng.integers(1, 999, L).tolist(),
                     act=[400] * L, grad=rng.integers(1, 10**6, L).tolist())
    for sched in (0, 1):
        ends = {}
        for dp in (1, 2, 8):
            cl = mk_cluster(dp * 4, g=1 << 20, alpha=(50, 50), beta=(200, 200))
            r = one(oracle_mod, costs, cl, (dp, 1, 4, 5, sched, None), timeline=True)
            ends[dp] = (r["end"].copy(), int(r["batch_ns"][0]), r["comm_busy_ns"].copy())
            if dp > 1:      # the single trailing all-reduce starts when the device's last backward ends
                assert np.array_equal(r["ar_window"][0], r["end"][1, :, 4])
            else:
                assert (r["ar_window"] == -1).all()
        assert np.array_equal(ends[1][0], ends[2][0]) and np.array_equal(ends[1][0], ends[8][0])
        G = [int(costs["grad_bytes"][0, 2 * s:2 * s + 2].sum()) for s in range(4)]
        for dp in (2, 8):
            ar = [50 + (2 * (dp - 1) * g) // (dp * 200) for g in G]
            want = max(int(ends[1][0][1, s, 4]) + ar[s] for s in range(4))
            assert ends[dp][1] == want
            assert list(ends[dp][2] - ends[1][2]) == ar


def test_async_schedule_is_dapple_without_the_global_sync(oracle_mod):
    """Sec. 7 (new algorithms): an asynchronous pipeline keeps the schedule and drops the global
    synchronisation event, which is the gradient all-reduce."""
    L = 8
    rng = np.random.default_rng(4)
    costs = mk_costs(rng.integers(1, 999, L).tolist(), rng.integers(1, 999, L).tolist(),
                     act=[400] * L, grad=rng.integers(1, 10**6, L).tolist())
    for bucket in (0, 3000):
        cl = mk_cluster(16, g=1 << 20, alpha=(50, 50), beta=(200, 200), bucket=bucket)
        sync = one(oracle_mod, costs, cl, (4, 1, 4, 6, 1, None), timeline=True)
        asyn = one(oracle_mod, costs, cl, (4, 1, 4, 6, 2, None), timeline=True)
        assert int(asyn["status"][0]) == 0
        # same device lists up to the all-reduce events
        assert np.array_equal(sync["start"], asyn["start"]) and np.array_equal(sync["end"], asyn["end"])
        assert (asyn["ar_window"] == -1).all() and (sync["ar_window"] >= 0).all()
        # the iteration ends with the last backward, and no all-reduce is accounted
        assert int(asyn["batch_ns"][0]) == int(asyn["end"].max()) < int(sync["batch_ns"][0])
        assert np.array_equal(asyn["comp_busy_ns"], sync["comp_busy_ns"])
        assert (asyn["comm_busy_ns"] < sync["comm_busy_ns"]).all()
        n_task, n_p2p = 2 * 6 * 4, 2 * 6 * 3
        assert int(asyn["num_events"][0]) == n_task + n_p2p
    # with one replica (no gradient exchange) the two schedules are the same thing
    cl = mk_cluster(4, g=1 << 20, alpha=(50, 50), beta=(200, 200))
    a = one(oracle_mod, costs, cl, (1, 1, 4, 6, 1, None))
    b = one(oracle_mod, costs, cl, (1, 1, 4, 6, 2, None))
    for k in ("batch_ns", "num_events", "comp_busy_ns", "comm_busy_ns"):
        assert np.array_equal(a[k], b[k])
    # unknown schedules stay invalid
    assert int(one(oracle_mod, costs, cl, (1, 1, 4, 6, 5, None))["status"][0]) == 1


# ----------------------------------------------------------------------------- interleaved schedule

def interleaved_order(pp, v, m, d):
    """Device d's task order under the interleaved schedule, from its definition: forward slot i is
    chunk (i mod pp v) / pp, micro-batch (i / (pp v)) pp + i mod pp; backward slot i the mirrored
    chunk; 2 (pp - d - 1) + (v - 1) pp warm-up forwards, then forward / backward in turn."""
    n = m * v

    def fwd(i):
        g, w = divmod(i, pp * v)
        return (w // pp, g * pp + w % pp)

    def bwd(i):
        g, w = divmod(i, pp * v)
        return (v - 1 - w // pp, g * pp + w % pp)
    W = min((pp - d - 1) * 2 + (v - 1) * pp, n)
    order = [("F",) + fwd(i) for i in range(W)]
    for i in range(n - W):
        order.append(("F",) + fwd(W + i))
        order.append(("B",) + bwd(i))
    order += [("B",) + bwd(i) for i in range(n - W, n)]
    return order


def interleaved_longest_path(pp, v, m, Fd, Bd, pf, pb):
    """End of every task (kind, virtual stage, micro-batch) by relaxation over the explicit graph."""
    S = pp * v
    preds = {}
    for d in range(pp):
        order = interleaved_order(pp, v, m, d)
        assert len(set(order)) == 2 * m * v == len(order)
        for i, (kd, c, j) in enumerate(order):
            k = c * pp + d
            p = []
            if i > 0:
                pk, pc, pj = order[i - 1]
                p.append(((pk, pc * pp + d, pj), 0))
            if kd == "F" and k > 0:
                p.append((("F", k - 1, j), pf[k - 1]))
            if kd == "B" and k < S - 1:
                p.append((("B", k + 1, j), pb[k + 1]))
            if kd == "B" and k == S - 1:
                p.append((("F", k, j), 0))
            preds[(kd, k, j)] = p
    dur = lambda n: Fd[n[1]] if n[0] == "F" else Bd[n[1]]
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
    return start, {n: start[n] + dur(n) for n in preds}


def test_interleaved_uniform_closed_form(oracle_mod):
    """Equal chunks, no p2p: the bubble of the interleaved schedule is (pp - 1)(tF + tB) / v for
    per-device times tF, tB (Narayanan et al., SC 2021), so batch = m (tF + tB) + (pp - 1)(tF + tB) / v."""
    for pp, v, groups in [(2, 2, 1), (4, 2, 2), (4, 4, 3), (8, 2, 1), (2, 3, 4), (3, 5, 2)]:
        m, S = pp * groups, pp * v
        f, b = 6, 10                                     # per chunk
        costs = mk_costs([f] * S, [b] * S, act=[0] * S)
        cl = mk_cluster(pp, g=1 << 20, alpha=(0, 0), beta=(1, 1))
        r = one(oracle_mod, costs, cl, (1, 1, pp, m, 3, None, v))
        assert int(r["status"][0]) == 0
        assert int(r["batch_ns"][0]) == m * v * (f + b) + (pp - 1) * (f + b)
        assert list(r["comp_busy_ns"]) == [m * v * (f + b)] * pp
        assert int(r["num_events"][0]) == 2 * m * S + 2 * m * (S - 1)
        # fewer bubbles than Dapple with the same devices and layers (v times thicker stages)
        costs1 = mk_costs([f * v] * pp, [b * v] * pp, act=[0] * pp)
        r1 = one(oracle_mod, costs1, cl, (1, 1, pp, m, 1, None))
        assert int(r1["batch_ns"][0]) == (m + pp - 1) * v * (f + b) >= int(r["batch_ns"][0])


def test_interleaved_against_task_graph(oracle_mod):
    rng = np.random.default_rng(41)
    for trial in range(250):
        pp = int(rng.integers(1, 6))
        v = int(rng.integers(1, 5))
        m = pp * int(rng.integers(1, 4))
        S = pp * v
        L = S + int(rng.integers(0, 4))
        cuts = sorted(rng.choice(np.arange(1, L), size=S - 1, replace=False).tolist())
        bnd = [0] + cuts + [L]
        fc = rng.integers(0, 40, L).tolist()
        bc = rng.integers(0, 60, L).tolist()
        act = (rng.integers(0, 9, L) * 5).tolist()
        dp = int(rng.choice([1, 2]))
        blocking = int(rng.integers(0, 2))
        costs = mk_costs(fc, bc, act=act, grad=[100] * L)
        cl = mk_cluster(dp * pp, g=1 << 20, alpha=(2, 0), beta=(5, 1), blocking=blocking)
        r = one(oracle_mod, costs, cl, (dp, 1, pp, m, 3, bnd, v), timeline=True)
        assert int(r["status"][0]) == 0
        pf = [2 + act[bnd[k + 1] - 1] // 5 for k in range(S - 1)] + [0]
        pb = [0] + [2 + act[bnd[k] - 1] // 5 for k in range(1, S)]
        F, B = _stage_sums(fc, bnd), _stage_sums(bc, bnd)
        if blocking:
            start, end = interleaved_longest_path(pp, v, m, [a + b for a, b in zip(F, pf)],
                                                  [a + b for a, b in zip(B, pb)], [0] * S, [0] * S)
        else:
            start, end = interleaved_longest_path(pp, v, m, F, B, pf, pb)
        for (k_, vs, j), val in end.items():
            kd = 0 if k_ == "F" else 1
            assert r["end"][kd, vs, j] == val, (trial, k_, vs, j)
            assert r["start"][kd, vs, j] == start[(k_, vs, j)]
        G = [100 * sum(bnd[c * pp + d + 1] - bnd[c * pp + d] for c in range(v)) for d in range(pp)]
        ar = [0 if dp == 1 else 2 + (2 * (dp - 1) * g) // (dp * 5) for g in G]
        dev_end = [max(val for (k_, vs, j), val in end.items() if vs % pp == d) for d in range(pp)]
        assert r["batch_ns"][0] == max(dev_end[d] + ar[d] for d in range(pp))
        for d in range(pp):                       # all-reduce window of every device in the dump
            assert r["ar_window"][0][d] == (dev_end[d] if dp > 1 else -1)
            assert r["ar_window"][1][d] == (dev_end[d] + ar[d] if dp > 1 else -1)
        for d in range(pp):
            comm = m * sum(pf[c * pp + d] + pb[c * pp + d] for c in range(v)) + ar[d]
            assert r["comm_busy_ns"][d] == comm
            assert r["comp_busy_ns"][d] == m * sum(F[c * pp + d] + B[c * pp + d] for c in range(v))


def test_interleaved_link_classes_follow_the_devices(oracle_mod):
    """Boundaries between virtual stages connect devices: with 2 ranks per device and 4 ranks per node,
    devices 0,1 | 2,3 sit on two nodes; 0->1 and 2->3 are intra-node, 1->2 and the edge from the last
    device back to the first (chunk c to chunk c + 1) are inter-node."""
    pp, v, m, S = 4, 2, 4, 8
    costs = mk_costs([0] * S, [0] * S, act=[200] * S, tps=(2,), grad=[0] * S)
    cl = mk_cluster(8, g=4)                            # alpha 5000 / 10000 ns, beta 200 / 25 B per ns
    r = one(oracle_mod, costs, cl, (1, 2, pp, m, 3, None, v))
    assert int(r["status"][0]) == 0
    intra, inter = 5000 + 200 // 200, 10_000 + 200 // 25
    edge = [intra, inter, intra, inter, intra, inter, intra]          # boundaries k | k+1 for k = 0..6
    pf = edge + [0]
    pb = [0] + edge
    want = [m * sum(pf[c * pp + d] + pb[c * pp + d] for c in range(v)) for d in range(pp)]
    assert list(r["comm_busy_ns"]) == want
    # four devices on one node hold 16 virtual stages: every boundary stays inside the node
    costs = mk_costs([0] * 16, [0] * 16, act=[200] * 16, grad=[0] * 16)
    r = one(oracle_mod, costs, mk_cluster(4, g=8), (1, 1, 4, 4, 3, None, 4))
    per_dev = [4 * (2 * 4 - (1 if d == 3 else 0) - (1 if d == 0 else 0)) * intra for d in range(4)]
    assert list(r["comm_busy_ns"]) == per_dev


def test_interleaved_validity_rules(oracle_mod):
    costs = mk_costs([5] * 12, [7] * 12)
    cl = mk_cluster(4, g=1 << 20)
    ok = lambda row: int(one(oracle_mod, costs, cl, row)["status"][0])
    assert ok((1, 1, 4, 8, 3, None, 3)) == 0
    assert ok((1, 1, 4, 6, 3, None, 3)) == 1           # m is not a multiple of pp
    assert ok((1, 1, 4, 8, 3, None, 4)) == 1           # 16 virtual stages, 12 layers
    assert ok((1, 1, 4, 8, 3, None, 0)) == 1
    assert ok((1, 1, 4, 8, 3, list(range(13)), 3)) == 0
    assert ok((1, 1, 4, 8, 3, [0, 3, 6, 9, 12], 3)) == 1     # boundaries of 4 parts where 12 are needed
    cl2 = mk_cluster(4, g=1 << 20, blocking=2)                  # link queues are modelled for this schedule too
    assert int(one(oracle_mod, costs, cl2, (1, 1, 4, 8, 3, None, 3))["status"][0]) == 0
    # nothing but the layer count bounds the number of virtual stages, nothing bounds the micro-batches
    many = mk_costs([5] * 200, [7] * 200)
    assert int(one(oracle_mod, many, cl, (1, 1, 4, 8, 3, None, 50))["status"][0]) == 0      # 200 virtual stages
    assert int(one(oracle_mod, many, cl, (1, 1, 4, 8, 3, None, 51))["status"][0]) == 1      # 204 > 200 layers
    r = one(oracle_mod, costs, mk_cluster(1), (1, 1, 1, (1 << 16) + 3, 1, None))
    assert int(r["status"][0]) == 0 and int(r["batch_ns"][0]) == ((1 << 16) + 3) * 12 * 12
    # one chunk per device is a valid degenerate case: Dapple's order with a warm-up twice as deep,
    # which hides the p2p latencies that Dapple's steady state leaves exposed
    a = one(oracle_mod, costs, cl, (1, 1, 4, 8, 3, None, 1))
    b = one(oracle_mod, costs, cl, (1, 1, 4, 8, 1, None))
    assert int(a["status"][0]) == 0 and int(a["batch_ns"][0]) <= int(b["batch_ns"][0])
    assert np.array_equal(a["comp_busy_ns"], b["comp_busy_ns"]) and np.array_equal(a["comm_busy_ns"], b["comm_busy_ns"])


# ----------------------------------------------------------------------------- paper facts

def test_paper_grid_has_15_settings():
    """Sec. 6: sizes 1,2,4,8,16 per dimension on 16 GPUs leave 15 valid (MP, PP) settings."""
    t = enumerate_triples(16, (1, 2, 4, 8, 16), 16)
    assert len(t) == 15
    assert all(d * a * p == 16 for d, a, p in t)
    w = make_workload("gpt24")
    assert w.C == 15 * 32 * 2


def test_paper_2m4p1d_has_32_stage_tasks(oracle_mod):
    """Sec. 5.4: "2m4p1d" with 4 micro-batches has 32 forward and backward stage-tasks, 4 + 4 per stage."""
    L = 8
    costs = mk_costs([10] * L, [20] * L, fa=[1] * L, ba=[1] * L, act=[0] * L, tps=(2,))
    r = one(oracle_mod, costs, mk_cluster(8), (1, 2, 4, 4, 1, None), timeline=True)
    assert r["start"].size == 32 and (r["start"] >= 0).all()
    assert r["num_events"][0] == 32 + 2 * 4 * 3
    assert r["start"][0, 0, 0] == 0                 # origin = start of the first stage's first event


def test_workload_sizes():
    assert make_workload("gpt48").C == 5888
    w = make_workload("gpt96")
    assert w.C == 102400 and w.cluster["dp_bucket_bytes"] == 25 << 20
    assert len(w.meta["triples"]) == 28


# ----------------------------------------------------------------------------- status / search

def test_invalid_and_range_status(oracle_mod):
    costs = mk_costs([10] * 4, [20] * 4, tps=(1,))
    rows = [
        (1, 1, 2, 4, 1, None),          # ok
        (2, 1, 2, 4, 1, None),          # dp*tp*pp != N
        (1, 2, 1, 4, 1, None),          # tp without variant (and product ok)
        (1, 1, 2, 0, 1, None),          # m < 1
        (1, 1, 2, 4, 1, [0, 0, 4]),     # empty stage
        (1, 1, 2, 4, 1, [0, 2, 3]),     # does not end at L
        (1, 1, 2, 4, 5, None),          # unknown schedule
        (1, 1, 2, 4, 0, [0, 1, 4]),     # ok
    ]
    r = oracle_mod.simulate(mk(costs, mk_cluster(2), rows))
    assert list(r["status"]) == [0, 1, 1, 1, 1, 1, 1, 0]
    assert all(r["batch_ns"][i] == INT64_MAX for i in range(1, 7))
    assert list(r["stage_off"]) == [0, 2, 2, 2, 2, 2, 2, 2, 4]
    # pp > L
    r = oracle_mod.simulate(mk(costs, mk_cluster(8), [(1, 1, 8, 1, 0, None)]))
    assert r["status"][0] == 1
    # 2^53 guard on m * (sum of all task and p2p durations)
    big = mk_costs([1 << 50] * 4, [1 << 50] * 4)
    r = oracle_mod.simulate(mk(big, mk_cluster(2), [(1, 1, 2, 1, 1, None), (1, 1, 2, 2, 1, None)]))
    assert list(r["status"]) == [2, 2]
    ok = mk_costs([1 << 48] * 4, [1 << 48] * 4)
    r = oracle_mod.simulate(mk(ok, mk_cluster(2), [(1, 1, 2, 1, 1, None), (1, 1, 2, 4, 1, None)]))
    assert list(r["status"]) == [0, 2]


def test_search_matches_python(oracle_mod):
    rng = np.random.default_rng(4)
    for trial in range(50):
        n = int(rng.integers(1, 200))
        b = rng.integers(1, 1 << 52, n)
        if trial % 3 == 0:
            b[rng.integers(0, n, n // 2 + 1)] = b[0]          # ties
        bad = rng.random(n) < 0.2
        b[bad] = INT64_MAX
        wgt = rng.integers(1, 1 << 20, n)
        valid = [i for i in range(n) if b[i] != INT64_MAX]
        i0, v0 = oracle_mod.search(b, None, 0)
        i1, v1 = oracle_mod.search(b, wgt, 1)
        if not valid:
            assert (i0, v0) == (-1, INT64_MAX) and i1 == -1
            continue
        want0 = min(valid, key=lambda i: (int(b[i]), i))
        from fractions import Fraction
        want1 = min(valid, key=lambda i: (Fraction(int(b[i]), int(wgt[i])), i))
        assert (i0, v0) == (want0, int(b[want0]))
        assert (i1, v1) == (want1, int(b[want1]))
