"""Pins of the oracle for the steps in front of event-flow generation (Sec. 4.1 event generator,
Sec. 4.2 profiling events).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle.ingest import comm_event_times, dedup_events
from workloads import make_comm_profiles, make_operator_records


def _i32(x): return np.asarray(x, dtype=np.int32)
def _i64(x): return np.asarray(x, dtype=np.int64)


# ---- Sec. 4.2 --------------------------------------------------------------------------

def test_p2p_is_min_of_send_and_recv():
    e = comm_event_times(_i32([0, 0, 0]), _i32([2, 2, 2]), _i64([700, 300, 5]), _i64([300, 700, 5]))
    assert e.tolist() == [300, 300, 5]


def test_allreduce_up_to_8_devices_is_the_profile_itself():
    for n in range(1, 9):
        assert comm_event_times(_i32([1]), _i32([n]), _i64([123456]), _i64([0])).tolist() == [123456]


def test_allreduce_rescale_is_the_ratio_of_ring_volumes():
    # Sec. 4.2: per-device volume 2(N-1)P/N; the 8-device profile is scaled by volume(N)/volume(8)
    P = 7 * 3 * 5 * 11 * 13 * 64            # divisible by many N, so that the volumes are integers
    for n in (9, 12, 16, 24, 64, 1024, 1536):
        vol_n, vol_8 = Fraction(2 * (n - 1) * P, n), Fraction(2 * 7 * P, 8)
        t8 = 10 ** 9
        want = int(Fraction(t8) * vol_n / vol_8)        # truncation
        assert comm_event_times(_i32([1]), _i32([n]), _i64([t8]), _i64([0])).tolist() == [want]
    # a bandwidth-only link (time = volume / beta): the rescaled 8-device time is the N-device time
    beta = 1
    for n in (16, 48, 112):
        t8 = 2 * 7 * P // 8 // beta
        tn = 2 * (n - 1) * P // n // beta
        assert 2 * (n - 1) * P % n == 0
        assert comm_event_times(_i32([1]), _i32([n]), _i64([t8]), _i64([0])).tolist() == [tn]


def test_allreduce_rescale_limit_and_monotonicity():
    t8 = 7 * 10 ** 12
    vals = comm_event_times(_i32([1] * 6), _i32([9, 10, 100, 10 ** 4, 10 ** 6, 2 ** 31 - 1]), _i64([t8] * 6), _i64([0] * 6))
    assert all(a <= b for a, b in zip(vals[:-1], vals[1:]))
    assert vals[0] == t8 * 8 * 8 // (7 * 9)
    assert vals[-1] <= t8 * 8 // 7 and t8 * 8 // 7 - vals[-1] <= t8 * 8 // 7 // 10 ** 9 + 1     # tends to 8/7 t8


def test_large_times_do_not_wrap():
    t8 = (1 << 61) + 12345
    n = 1000
    assert comm_event_times(_i32([1]), _i32([n]), _i64([t8]), _i64([0])).tolist() == [t8 * 8 * 999 // 7000]


def test_invalid_profile_records():
    e = comm_event_times(_i32([2, 1, 1, 0, 0, -1]), _i32([4, 0, 4, 2, 2, 2]), _i64([5, 5, -1, -1, 5, 5]), _i64([5, 5, 5, 5, -2, 5]))
    assert e.tolist() == [-1, -1, -1, -1, -1, -1]


# ---- Sec. 4.1 --------------------------------------------------------------------------

def _brute_partition(records):
    n = len(records)
    return {(i, j) for i in range(n) for j in range(n) if (records[i] == records[j]).all()}


def test_dedup_small_against_all_pairs():
    rng = np.random.default_rng(5)
    rec = rng.integers(0, 3, size=(60, 3)).astype(np.int64)
    eid, rep = dedup_events(rec)
    assert {(i, j) for i in range(60) for j in range(60) if eid[i] == eid[j]} == _brute_partition(rec)
    # numbered by first occurrence; rep is that occurrence
    firsts = [int(np.nonzero(eid == e)[0][0]) for e in range(len(rep))]
    assert firsts == sorted(firsts) and firsts == rep.tolist()
    assert eid.max() + 1 == len(rep) == len(np.unique(rec, axis=0))


def test_dedup_agrees_with_row_unique_on_a_large_draw():
    rec = make_operator_records(200_000, 3000)
    eid, rep = dedup_events(rec)
    uniq, first, inv = np.unique(rec, axis=0, return_index=True, return_inverse=True)
    order = np.argsort(first)                       # unique rows by first occurrence
    rank = np.empty_like(order); rank[order] = np.arange(len(order))
    assert (eid == rank[inv.reshape(-1)]).all()
    assert (rep == first[order]).all()


def test_dedup_special_cases():
    eid, rep = dedup_events(np.zeros((0, 4), dtype=np.int64))
    assert len(eid) == 0 and len(rep) == 0
    eid, rep = dedup_events(np.full((17, 2), 9, dtype=np.int64))
    assert eid.tolist() == [0] * 17 and rep.tolist() == [0]
    rec = np.arange(10, dtype=np.int64).reshape(10, 1)
    eid, rep = dedup_events(rec)
    assert eid.tolist() == list(range(10)) and rep.tolist() == list(range(10))
    # records that differ only in the last word (the intra-/inter-node attribute) are two events
    eid, _ = dedup_events(_i64([[1, 2, 0], [1, 2, 1], [1, 2, 0]]))
    assert eid.tolist() == [0, 1, 0]


def test_profiled_once_per_event():
    # Sec. 3.2 / 4.1: identical operators are profiled a single time, so there are as many profiling jobs as events
    rec = make_operator_records(50_000, 400)
    eid, rep = dedup_events(rec)
    assert len(rep) <= 400 and (rec[rep[eid]] == rec).all()


# ---- bubble analysis of a timeline (Sec. 3.2, Sec. 5) ------------------------------------------

def _timeline_of(oracle_mod, costs, cluster, row):
    from helpers import mk
    return oracle_mod.simulate(mk(costs, cluster, [row]), timeline=True)


@pytest.mark.parametrize("sched", [0, 1, 2])
def test_bubbles_account_for_all_idle_time(oracle_mod, sched):
    from helpers import mk_cluster, mk_costs
    from oracle.bubbles import device_order, idle_before
    rng = np.random.default_rng(8 + sched)
    L = 12
    for pp, m in [(1, 1), (1, 5), (2, 4), (3, 7), (4, 2), (6, 6), (12, 3)]:
        costs = mk_costs(rng.integers(1, 900, L).tolist(), rng.integers(1, 900, L).tolist(), act=[3000] * L)
        r = _timeline_of(oracle_mod, costs, mk_cluster(pp, alpha=(40, 40), beta=(10, 10)), (1, 1, pp, m, sched, None))
        st, en = r["start"], r["end"]
        idle = idle_before(st, en, sched)
        assert (idle >= 0).all()
        for s in range(pp):
            order = device_order(pp, m, sched, s)
            assert sorted(order) == sorted([(k, j) for k in (0, 1) for j in range(m)])       # every task once
            # idle + busy = the time at which the device finishes its last task
            busy = int((en[:, s, :] - st[:, s, :]).sum())
            assert int(idle[:, s, :].sum()) + busy == int(en[:, s, :].max())
            # without zero-length tasks the device order is the order of the start times
            by_time = sorted([(int(st[k, s, j]), k, j) for k in (0, 1) for j in range(m)])
            assert [(k, j) for _, k, j in by_time] == order
        # the first stage never waits for its first forward; the last stage's first backward follows
        # its own forward of the same micro-batch under Dapple
        assert idle[0, 0, 0] == 0


def test_bubbles_of_the_interleaved_schedule(oracle_mod):
    """The same accounting over virtual stages: every task of a device once, no negative idle time,
    idle + busy = end of the device's last task, and (positive durations) the list order is the
    order of the start times.  With one chunk the list is the Dapple list with the longer warm-up."""
    from helpers import mk_cluster, mk_costs
    from oracle.bubbles import device_order_interleaved, idle_before
    rng = np.random.default_rng(77)
    L = 24
    for pp, v, groups in [(1, 1, 3), (1, 4, 2), (2, 2, 1), (2, 3, 4), (3, 2, 2), (4, 3, 1), (4, 6, 3), (6, 4, 2), (8, 1, 2)]:
        m = pp * groups
        costs = mk_costs(rng.integers(1, 900, L).tolist(), rng.integers(1, 900, L).tolist(), act=[3000] * L)
        r = _timeline_of(oracle_mod, costs, mk_cluster(pp, alpha=(40, 40), beta=(10, 10)), (1, 1, pp, m, 3, None, v))
        assert r["status"][0] == 0
        st, en = r["start"], r["end"]
        assert st.shape == (2, pp * v, m)
        idle = idle_before(st, en, 3, v)
        assert (idle >= 0).all()
        for d in range(pp):
            order = device_order_interleaved(pp, m, v, d)
            mine = [(k, c * pp + d, j) for k in (0, 1) for c in range(v) for j in range(m)]
            assert sorted(order) == sorted(mine)
            rows = [c * pp + d for c in range(v)]
            busy = int((en[:, rows, :] - st[:, rows, :]).sum())
            assert int(idle[:, rows, :].sum()) + busy == int(en[:, rows, :].max())
            by_time = sorted([(int(st[k, vs, j]), k, vs, j) for k, vs, j in mine])
            assert [(k, vs, j) for _, k, vs, j in by_time] == order
            if v == 1:
                w = min(2 * (pp - d - 1), m)
                assert order[:w] == [(0, d, j) for j in range(w)] and (w == m or order[w + 1] == (1, d, 0))
        assert idle[0, 0, 0] == 0


def test_bubbles_of_the_hand_unrolled_pipeline(oracle_mod):
    """pp = 2, m = 4, Dapple, uniform stages F = 10, B = 20, p2p c = 3 (the timeline of
    tests/golden/pipeline_pp2_m4.txt with numbers put in): stage 1 idles F + c before its first
    forward; stage 0 idles c + B + c between its second forward and its first backward."""
    from helpers import mk_cluster, mk_costs
    from oracle.bubbles import idle_before
    costs = mk_costs([10, 10], [20, 20], act=[30, 30])
    r = _timeline_of(oracle_mod, costs, mk_cluster(2, alpha=(0, 0), beta=(10, 10)), (1, 1, 2, 4, 1, [0, 1, 2]))
    idle = idle_before(r["start"], r["end"], 1)
    F, B, c = 10, 20, 3
    assert idle[0, 1, 0] == F + c                       # stage 1 waits for the first activation
    assert idle[0, 0, 0] == 0 and idle[0, 0, 1] == 0    # stage 0: warm-up forward, then F1 back to back
    assert idle[1, 0, 0] == (F + c + F + B + c) - 2 * F  # B0 on stage 0 arrives after stage 1's F0, B0 and two sends
    assert int(idle.sum()) > 0
