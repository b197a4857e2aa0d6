"""Pins of the bucketed gradient all-reduce of the interleaved and the explicit schedules (a device
holds several virtual stages and fills its buckets across them).  CPU only.  The bucketed
all-reduce is this library's extension of the data-parallel modelling step (Sec. 4.3: one
all-reduce event at the end of each device's list); none of the expected values below comes from
the routine under test:

 * a device with two chunks worked by hand (bucket of 200 and of 100 bytes);
 * the lists of GPipe and Dapple written out as explicit schedules must give what the oracle's
   routine for the built-in schedules gives with the same buckets (two routines, one answer), and
   the interleaved order written out as lists what the interleaved routine gives;
 * properties on random cases: buckets change nothing before the device's last gradients (task
   start and end times equal those without buckets); the number of all-reduce events and their busy
   time follow from the device's gradient bytes alone; a bucket larger than all gradients gives the
   single trailing event; an explicit graph of the bucket chain (ready times from the dumped task
   starts, one queue per device) gives every device's all-reduce window.
"""
import numpy as np

from helpers import mk, mk_cluster, mk_costs
from test_explicit_schedule_pins import rand_costs, same_result, with_schedules
from workloads import Workload, subset
from workloads.schedules import (bidirectional_lists, bidirectional_stages, chain, dapple_lists, gpipe_lists,
                                 interleaved_lists, interleaved_stages, pack_schedule)


def ar_ns(alpha, beta, n, nbytes):
    return alpha + (2 * (n - 1) * nbytes) // (n * beta)


def test_two_chunks_on_one_device_by_hand(oracle_mod):
    """pp = 1, two chunks (layer 0, layer 1), one micro-batch, dp = 2.  The activation between the
    chunks is a p2p event of alpha = 5 ns (no bytes): F0 0-10, F1 15-35, B1 35-75, B0 80-110.  Layer
    1's 250 bytes are there at 75, layer 0's 100 bytes at 110.  An all-reduce of b bytes over two
    ranks takes 5 + b / 10 ns."""
    costs = mk_costs([10, 20], [30, 40], grad=[100, 250])
    for bucket, windows, batch, nar in (
            # 250 >= 200: one bucket 75-100, 50 left; at 110: 150 left over after the last gradient: 110-130
            (200, (75, 130), 130, 2),
            # two buckets 75-90-105, 50 left; at 110: 150 -> one bucket 110-125, then the rest 125-135
            (100, (75, 135), 135, 4),
            # everything in one event after the last gradient: 350 bytes, 40 ns
            (1000, (110, 150), 150, 1)):
        cl = mk_cluster(2, g=8, alpha=(5, 7), beta=(10, 3), bucket=bucket)
        w = mk(costs, cl, [(2, 1, 1, 1, 3, [0, 1, 2], 2)])
        w.cand["chunks"] = np.asarray([2], np.int32)
        r = oracle_mod.simulate(w, timeline=True)
        assert r["status"][0] == 0
        assert r["batch_ns"][0] == batch, bucket
        assert (int(r["ar_window"][0][0]), int(r["ar_window"][1][0])) == windows, bucket
        assert r["num_events"][0] == 4 + 2 + nar                      # tasks, the two p2p events, the all-reduce events
        full, rest = divmod(350, bucket)
        busy = full * ar_ns(5, 10, 2, bucket) + (ar_ns(5, 10, 2, rest) if rest else 0)
        assert r["comm_busy_ns"][0] == busy + 10 and r["comp_busy_ns"][0] == 100
        assert r["start"][:, :, 0].tolist() == [[0, 15], [80, 35]] and r["end"][:, :, 0].tolist() == [[10, 35], [110, 75]]


def test_lists_of_the_built_in_schedules_with_buckets(oracle_mod):
    rng = np.random.default_rng(17)
    n_bucketed = 0
    for trial in range(240):
        pp = int(rng.integers(1, 7))
        v = int(rng.integers(1, 4))
        m = pp * int(rng.integers(1, 4)) if trial % 3 == 2 else int(rng.integers(1, 9))
        tp = int(rng.choice([1, 2]))
        dp = int(rng.choice([1, 2, 3]))
        L = pp * v + int(rng.integers(0, 5))
        costs = rand_costs(rng, L, tps=(1, 2))
        blocking = int(rng.integers(0, 3))
        bucket = int(rng.choice([1, 60, 250, 700, 10**6]))
        cl = mk_cluster(dp * tp * pp, g=int(rng.choice([1, 2, 4, 64])), alpha=(3, 11), beta=(5, 2), blocking=blocking,
                        bucket=bucket)
        if trial % 3 == 2:
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
        assert r["status"][0] == 0 and r["status"][1] == 0
        same_result(r, r, 0, 1, f"trial {trial}")
        a, b = (oracle_mod.simulate(subset(w, [c]), timeline=True) for c in (0, 1))
        assert np.array_equal(a["ar_window"], b["ar_window"]), trial
        assert np.array_equal(a["start"], b["start"]) and np.array_equal(a["end"], b["end"]), trial
        n_bucketed += int(dp > 1)
    assert n_bucketed > 100


def _devices(w, c):
    """(virtual stages of every device in the order of their last backward, layer range of every
    virtual stage) of interleaved candidate c."""
    pp, v = int(w.cand["pp"][c]), int(w.cand["chunks"][c])
    po = int(w.cand["part_off"][c])
    S = pp * v
    bnd = w.cand["part_pool"][po:po + S + 1].astype(int) if po >= 0 else np.asarray([(k * w.L) // S for k in range(S + 1)])
    return [[ch * pp + d for ch in range(v - 1, -1, -1)] for d in range(pp)], bnd


def test_bucket_chain_of_interleaved_candidates_from_the_dump(oracle_mod):
    """Every device's all-reduce window, event count and busy time, rebuilt outside the routine: the
    ready time of a layer's gradient = start of that chunk's backward of the last micro-batch (read
    from the dump) + the backward events from the chunk's last layer down to that layer (summed here
    from the cost table); buckets fill in that order and queue on one stream per device."""
    rng = np.random.default_rng(23)
    checked = 0
    for trial in range(120):
        pp = int(rng.integers(1, 6))
        v = int(rng.integers(1, 4))
        m = pp * int(rng.integers(1, 4))
        dp = int(rng.choice([2, 3, 4]))
        L = pp * v + int(rng.integers(0, 6))
        costs = rand_costs(rng, L)
        blocking = int(rng.integers(0, 3))
        bucket = int(rng.choice([40, 150, 400, 2000]))
        alpha, beta = (3, 11), (5, 2)
        g = int(rng.choice([1, 2, 64]))
        cl = mk_cluster(dp * pp, g=g, alpha=alpha, beta=beta, blocking=blocking, bucket=bucket)
        S = pp * v
        bnd = [0] + sorted(rng.choice(np.arange(1, L), S - 1, replace=False).tolist()) + [L]
        w = mk(costs, cl, [(dp, 1, pp, m, 3, bnd, v)])
        w.cand["chunks"] = np.asarray([v], np.int32)
        r = oracle_mod.simulate(w, timeline=True)
        w0 = Workload("no buckets", w.costs, dict(w.cluster, dp_bucket_bytes=0), w.cand)
        r0 = oracle_mod.simulate(w0, timeline=True)
        assert r["status"][0] == 0
        # buckets change no task
        assert np.array_equal(r["start"], r0["start"]) and np.array_equal(r["end"], r0["end"])
        k_link = 0 if dp <= g else 1
        devs, bnd = _devices(w, 0)
        bc, grad = w.costs["bwd_comp_ns"][0], w.costs["grad_bytes"][0]
        a2a = w.costs["a2a_bytes"][0] if "a2a_bytes" in w.costs else np.zeros(L, np.int64)
        assert not np.any(a2a)                        # rand_costs has no all-to-all: a backward layer event is bc alone (tp = 1)
        last_end = 0
        n_ar = 0
        for d, stages in enumerate(devs):
            free, acc, first, busy = 0, 0, -1, 0
            pend = sum(int(bnd[k + 1] - bnd[k]) for k in stages)
            for k in stages:
                t = int(r["start"][1, k, m - 1])
                for l in range(int(bnd[k + 1]) - 1, int(bnd[k]) - 1, -1):
                    t += int(bc[l])
                    acc += int(grad[l]); pend -= 1
                    while acc >= bucket or (pend == 0 and acc > 0):
                        nbytes = min(acc, bucket)
                        st = max(free, t)
                        dur = ar_ns(alpha[k_link], beta[k_link], dp, nbytes)
                        free = st + dur
                        busy += dur; n_ar += 1
                        first = st if first < 0 else first
                        acc -= nbytes
            assert int(r["ar_window"][0][d]) == first and int(r["ar_window"][1][d]) == (free if first >= 0 else -1), (trial, d)
            assert r["comm_busy_ns"][d] - r0["comm_busy_ns"][d] == busy - (int(r0["ar_window"][1][d]) - int(r0["ar_window"][0][d]) if r0["ar_window"][0][d] >= 0 else 0)
            G = sum(int(grad[bnd[k]:bnd[k + 1]].sum()) for k in stages)
            if first >= 0:
                assert busy == (G // bucket) * ar_ns(alpha[k_link], beta[k_link], dp, bucket) + \
                    (ar_ns(alpha[k_link], beta[k_link], dp, G % bucket) if G % bucket else 0)
            last_end = max(last_end, free)
            checked += 1
        assert r["batch_ns"][0] == max(last_end, int(r["end"].max()))
        assert r["num_events"][0] - r0["num_events"][0] == n_ar - int((r0["ar_window"][0][:pp] >= 0).sum())
    assert checked > 250


def test_a_bucket_larger_than_all_gradients_is_the_trailing_event(oracle_mod):
    rng = np.random.default_rng(29)
    for trial in range(60):
        pp = int(rng.integers(1, 6))
        v = int(rng.integers(1, 4))
        m = pp * int(rng.integers(1, 3))
        dp = int(rng.choice([2, 4]))
        L = pp * v + int(rng.integers(0, 4))
        costs = rand_costs(rng, L)
        blocking = int(rng.choice([0, 2]))            # with the send inside the task the last gradient precedes the end of the list
        S = pp * v
        bnd = [0] + sorted(rng.choice(np.arange(1, L), S - 1, replace=False).tolist()) + [L]
        res = []
        for bucket in (0, 10**9):
            cl = mk_cluster(dp * pp, g=int(rng.choice([1, 64])) if bucket == 0 else res_g, alpha=(3, 11), beta=(5, 2),
                            blocking=blocking, bucket=bucket)
            res_g = cl["gpus_per_node"]
            blk = pack_schedule(pp, interleaved_stages(pp, v), m, S, 1, interleaved_lists(pp, v, m))
            w = with_schedules(mk(costs, cl, [(dp, 1, pp, m, 3, bnd, v), (dp, 1, pp, m, 4, bnd, 0)]), [blk], [v, 0])
            res.append((oracle_mod.simulate(w), [oracle_mod.simulate(subset(w, [c]), timeline=True) for c in (0, 1)]))
        for c in (0, 1):
            same_result(res[0][0], res[1][0], c, c, f"trial {trial} candidate {c}")
            assert np.array_equal(res[0][1][c]["ar_window"], res[1][1][c]["ar_window"])


def test_a_stage_without_backward_gives_no_gradient_with_buckets(oracle_mod):
    """Three stages, each a pipeline of its own: stages 0 and 2 on device 0, stage 1 on device 1.
    Device 0 runs F(0), F(2), B(0); device 1 only F(1) (a schedule may stop there).  All-reduce over
    two ranks: 5 + bytes / 10 ns.
    Without buckets every device reduces the bytes of all its stages after its list: device 0
    120 + 60 bytes from 45 to 68, device 1 250 bytes from 20 to 50.
    With buckets of 50 bytes only stage 0 produces gradients: 120 bytes at 45, two buckets 45-55-65
    and the rest of 20 bytes 65-72; the stage without a backward neither adds bytes nor keeps the
    rest waiting; device 1 reduces nothing."""
    costs = mk_costs([10, 20, 5], [30, 40, 7], grad=[120, 250, 60])
    stages = [(0, 0, -1), (1, 1, -1), (0, 2, -1)]              # (device, part, stage before it)
    lists = [[(0, 0, 0), (0, 2, 0), (1, 0, 0)], [(0, 1, 0)]]   # (kind, stage, micro-batch)
    blk = pack_schedule(2, stages, 1, 3, 1, lists)
    for bucket, windows, batch, n_ar in ((0, [(45, 68), (20, 50)], 68, 2), (50, [(45, 72), (-1, -1)], 72, 3)):
        cl = mk_cluster(4, g=8, alpha=(5, 7), beta=(10, 3), bucket=bucket)
        w = with_schedules(mk(costs, cl, [(2, 1, 2, 1, 4, [0, 1, 2, 3], 0)]), [blk], [0])
        r = oracle_mod.simulate(w, timeline=True)
        assert r["status"][0] == 0
        assert [(int(r["ar_window"][0][d]), int(r["ar_window"][1][d])) for d in range(2)] == windows, bucket
        assert r["batch_ns"][0] == batch and r["num_events"][0] == 4 + n_ar


def test_replicas_enter_the_bucket_events(oracle_mod):
    """Two pipelines in opposite directions over the same devices: every device holds one stage of
    each, the all-reduce spans dp * 2 ranks.  Busy time and number of the bucket events from the
    device's bytes alone."""
    rng = np.random.default_rng(31)
    for trial in range(40):
        pp = int(rng.integers(2, 6))
        m = 2 * int(rng.integers(1, 4))
        dp = int(rng.choice([1, 2, 3]))
        L = pp + int(rng.integers(0, 4))
        costs = rand_costs(rng, L)
        bucket = int(rng.choice([50, 170, 900]))
        g = int(rng.choice([1, 4, 64]))
        alpha, beta = (3, 11), (5, 2)
        bnd = [0] + sorted(rng.choice(np.arange(1, L), pp - 1, replace=False).tolist()) + [L]
        stages = bidirectional_stages(pp)
        blk = pack_schedule(pp, stages, m, pp, 2, bidirectional_lists(pp, m))
        out = []
        for b in (0, bucket):
            cl = mk_cluster(dp * pp, g=g, alpha=alpha, beta=beta, bucket=b)
            w = with_schedules(mk(costs, cl, [(dp, 1, pp, m, 4, bnd, 0)]), [blk], [0])
            out.append(oracle_mod.simulate(w))
            assert out[-1]["status"][0] == 0
        ranks = 2 * dp
        k = 0 if ranks <= g else 1
        grad = costs["grad_bytes"][0]
        n_more = 0
        for d in range(pp):
            G = sum(int(grad[bnd[part]:bnd[part + 1]].sum()) for (dev, part, _prev) in stages if dev == d)
            if G == 0:
                continue
            full, rest = divmod(G, bucket)
            busy = full * ar_ns(alpha[k], beta[k], ranks, bucket) + (ar_ns(alpha[k], beta[k], ranks, rest) if rest else 0)
            assert out[1]["comm_busy_ns"][d] - out[0]["comm_busy_ns"][d] == busy - ar_ns(alpha[k], beta[k], ranks, G), (trial, d)
            n_more += full + (1 if rest else 0) - 1
        assert out[1]["num_events"][0] - out[0]["num_events"][0] == n_more
