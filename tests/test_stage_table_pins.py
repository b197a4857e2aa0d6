"""Pins of the oracle's stage table (oracle_stage_table: the composed events of every stage, summed
with plain loops over the stage's layers).  None of the expected values comes from that routine:

 * the Tiny example's p2p event 5000 + 4 MiB / 200 B/ns = 25 971 ns and its layer ranges;
 * every column separately against the oracle's discrete-event timeline of the same candidate run
   with one micro-batch in GPipe order (the DES executes layer events one by one and knows no
   stage sums): a forward task lasts FC + FA, a backward task BC + BA, the next stage starts PF
   after a forward ends, the previous stage PB after a backward ends, the all-reduce window is AR
   long, and with the other computation column zeroed the computation busy time is FC (or BC);
 * the busy-time identities of the analysis step on whole workloads:
   computation busy = m (FC + BC), communication busy = m (FA + BA + PF + PB) + AR.
"""
import numpy as np
import pytest

from helpers import mk, mk_cluster, mk_costs
from workloads import Workload, make_workload, subset


def test_tiny_golden_stage_events(oracle_mod):
    costs = mk_costs([1_000_000] * 4, [2_025_000] * 4, act=[4 << 20] * 4)
    w = mk(costs, mk_cluster(2), [(1, 1, 2, 4, 1, [0, 2, 4]), (1, 1, 2, 4, 0, None)])
    sim = oracle_mod.simulate(w)
    t = oracle_mod.stage_table(w, sim)
    assert t["tab"][0].tolist() == [2_000_000] * 4 and t["tab"][2].tolist() == [4_050_000] * 4
    assert t["tab"][1].tolist() == [0] * 4 and t["tab"][3].tolist() == [0] * 4
    assert t["tab"][4].tolist() == [25_971, 0, 25_971, 0]
    assert t["tab"][5].tolist() == [0, 25_971, 0, 25_971]
    assert t["tab"][6].tolist() == [0] * 4 and t["tab"][7].tolist() == [0] * 4
    assert t["layer_lo"].tolist() == [0, 2, 0, 2] and t["layer_hi"].tolist() == [2, 4, 2, 4]


def _columns_from_timelines(oracle_mod, w, c):
    """Columns of candidate c of workload w, each read off a discrete-event run."""
    one = subset(w, [c])
    one.cand["m"] = np.asarray([1], np.int32)
    sched = int(one.cand["schedule"][0])
    one.cand["schedule"] = np.asarray([2 if sched == 2 else 0], np.uint8)     # one micro-batch: the order is F then B anyway
    cl = dict(w.cluster); cl["dp_bucket_bytes"] = 0; cl["p2p_blocking"] = 0
    one = Workload("one", w.costs, cl, one.cand)
    r = oracle_mod.simulate(one, timeline=True)
    assert r["status"][0] == 0
    pp = int(one.cand["pp"][0])
    st, en = r["start"], r["end"]
    Fd = en[0, :, 0] - st[0, :, 0]
    Bd = en[1, :, 0] - st[1, :, 0]
    PF = np.zeros(pp, np.int64); PB = np.zeros(pp, np.int64)
    PF[:-1] = st[0, 1:, 0] - en[0, :-1, 0]             # nothing else can delay a stage's only forward
    PB[1:] = st[1, :-1, 0] - en[1, 1:, 0]
    AR = np.where(r["ar_window"][0] >= 0, r["ar_window"][1] - r["ar_window"][0], 0)
    zero_b = dict(w.costs); zero_b["bwd_comp_ns"] = np.zeros_like(w.costs["bwd_comp_ns"])
    zero_f = dict(w.costs); zero_f["fwd_comp_ns"] = np.zeros_like(w.costs["fwd_comp_ns"])
    FC = oracle_mod.simulate(Workload("zb", zero_b, cl, one.cand))["comp_busy_ns"]
    BC = oracle_mod.simulate(Workload("zf", zero_f, cl, one.cand))["comp_busy_ns"]
    return FC, Fd - FC, BC, Bd - BC, PF, PB, AR


def _check_against_timelines(oracle_mod, w, idx):
    w = subset(w, np.sort(np.asarray(idx)))
    idx = np.arange(w.C)
    sim = oracle_mod.simulate(w, nthreads=8)
    t = oracle_mod.stage_table(w, sim)
    so = sim["stage_off"]
    n = 0
    for c in idx:
        if sim["status"][c] != 0 or w.cand["schedule"][c] > 2:
            continue
        FC, FA, BC, BA, PF, PB, AR = _columns_from_timelines(oracle_mod, w, int(c))
        rows = slice(so[c], so[c + 1])
        for col, want in zip((0, 1, 2, 3, 4, 5, 7), (FC, FA, BC, BA, PF, PB, AR)):
            assert np.array_equal(t["tab"][col, rows], want), (w.name, int(c), col)
        # gradient bytes and layer ranges: the partition and a sum of the table's entries
        pp, tp = int(w.cand["pp"][c]), int(w.cand["tp"][c])
        v = int(np.nonzero(w.costs["variant_tp"] == tp)[0][0])
        po = int(w.cand["part_off"][c])
        bnd = w.cand["part_pool"][po:po + pp + 1].astype(int) if po >= 0 else [(s * w.L) // pp for s in range(pp + 1)]
        assert t["layer_lo"][rows].tolist() == list(bnd[:-1]) and t["layer_hi"][rows].tolist() == list(bnd[1:])
        assert t["tab"][6, rows].tolist() == [int(w.costs["grad_bytes"][v, bnd[s]:bnd[s + 1]].sum()) for s in range(pp)]
        n += 1
    return n


def test_every_column_against_discrete_event_timelines(oracle_mod):
    rng = np.random.default_rng(4)
    n = 0
    for name in ("gpt24", "gpt48", "gpt96", "hetero64"):
        w = make_workload(name, C=3000) if name == "hetero64" else make_workload(name)
        n += _check_against_timelines(oracle_mod, w, rng.choice(w.C, 40, replace=False))
    # ragged shapes: odd stage counts, several variants, all-to-all, zero entries, asynchronous schedule
    L = 30
    costs = mk_costs(rng.integers(0, 5000, (3, L)).tolist(), rng.integers(0, 9000, (3, L)).tolist(),
                     fa=rng.integers(1, 300, (3, L)).tolist(), ba=rng.integers(1, 300, (3, L)).tolist(),
                     act=(rng.integers(0, 100, (3, L)) * 64).tolist(), grad=rng.integers(0, 1 << 20, (3, L)).tolist(),
                     a2a=(rng.integers(0, 3, (3, L)) * 4096).tolist(), tps=(1, 2, 3))
    N = 2 * 3 * 5 * 7 * 8
    rows = []
    for _ in range(120):
        pp = int(rng.choice([d for d in range(1, 25) if N % d == 0]))
        tp = int(rng.choice([t for t in (1, 2, 3) if (N // pp) % t == 0]))
        bnd = [0] + np.sort(rng.choice(np.arange(1, L), pp - 1, replace=False)).tolist() + [L] if rng.random() < 0.6 else None
        rows.append((N // (pp * tp), tp, pp, int(rng.integers(1, 9)), int(rng.integers(0, 3)), bnd))
    for g in (1, 4, 16):
        w = mk(costs, mk_cluster(N, g=g), rows, name=f"ragged g={g}")
        n += _check_against_timelines(oracle_mod, w, np.arange(len(rows)))
    assert n > 400


@pytest.mark.parametrize("name", ["gpt24", "gpt48", "gpt96", "hetero64"])
def test_busy_time_identities(oracle_mod, name):
    """Analysis step: a device's busy time is the sum of the durations of its events."""
    w = make_workload(name, C=20000) if name == "hetero64" else make_workload(name)
    if name == "gpt96":
        w = subset(w, np.arange(0, w.C, 9))
        w.cluster["dp_bucket_bytes"] = 0              # one trailing all-reduce: its duration is the AR column
    sim = oracle_mod.simulate(w, nthreads=8)
    t = oracle_mod.stage_table(w, sim)["tab"]
    ok = sim["status"] == 0
    assert ok.all()
    m = np.repeat(w.cand["m"].astype(np.int64), w.cand["pp"])
    assert np.array_equal(sim["comp_busy_ns"], m * (t[0] + t[2]))
    assert np.array_equal(sim["comm_busy_ns"], m * (t[1] + t[3] + t[4] + t[5]) + t[7])


def test_candidates_without_a_stage_table_keep_zeros(oracle_mod):
    costs = mk_costs([5] * 12, [7] * 12, grad=[100] * 12)
    rows = [(2, 1, 4, 8, 3, None, 3), (2, 1, 4, 8, 1, None, 1), (3, 1, 4, 8, 1, None, 1)]
    w = mk(costs, mk_cluster(8), rows)
    sim = oracle_mod.simulate(w)
    assert sim["status"].tolist() == [0, 0, 1]
    t = oracle_mod.stage_table(w, sim)
    assert t["tab"].shape == (8, 8) and not t["tab"][:, :4].any() and t["tab"][0, 4:].tolist() == [15] * 4
