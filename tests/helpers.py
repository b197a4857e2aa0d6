"""Small builders shared by the tests (inputs only; no simulator arithmetic)."""
from __future__ import annotations

import numpy as np

from workloads import Workload


def mk_costs(fc, bc, fa=None, ba=None, act=None, grad=None, a2a=None, tps=(1,)):
    """Cost table from per-variant rows.  Each argument: list over variants of lists over layers,
    or a single list (then V = 1)."""
    def arr(x, default=0):
        if x is None:
            return None
        a = np.asarray(x, dtype=np.int64)
        if a.ndim == 1:
            a = a[None, :]
        return a
    fc = arr(fc)
    V, L = fc.shape
    def fill(x):
        a = arr(x)
        if a is None:
            return np.zeros((V, L), np.int64)
        if a.shape == (1, 1):
            return np.full((V, L), int(a[0, 0]), np.int64)
        assert a.shape == (V, L), (a.shape, V, L)
        return a
    assert len(tps) == V
    return {
        "L": L, "V": V, "variant_tp": np.asarray(tps, np.int32),
        "fwd_comp_ns": fc, "bwd_comp_ns": fill(bc),
        "fwd_comm_ns": fill(fa), "bwd_comm_ns": fill(ba),
        "act_bytes": fill(act), "grad_bytes": fill(grad), "a2a_bytes": fill(a2a),
    }


def mk_cluster(n, g=8, alpha=(5000, 10000), beta=(200, 25), bucket=0, blocking=0):
    return {"num_devices": int(n), "gpus_per_node": int(g), "alpha_ns": tuple(alpha),
            "beta_bytes_per_ns": tuple(beta), "dp_bucket_bytes": int(bucket), "p2p_blocking": int(blocking)}


def mk_cands(rows):
    """rows: list of (dp, tp, pp, m, schedule, bnd-or-None[, chunks])."""
    dp, tp, pp, m, sc, off, pool, ch = [], [], [], [], [], [], [], []
    for row in rows:
        (d, t, p, mm, s, bnd) = row[:6]
        ch.append(row[6] if len(row) > 6 else 1)
        dp.append(d); tp.append(t); pp.append(p); m.append(mm); sc.append(s)
        if bnd is None:
            off.append(-1)
        else:
            off.append(len(pool))
            pool.extend(int(b) for b in bnd)
    return {
        "dp": np.asarray(dp, np.int32), "tp": np.asarray(tp, np.int32),
        "pp": np.asarray(pp, np.int32), "m": np.asarray(m, np.int32),
        "schedule": np.asarray(sc, np.uint8), "part_off": np.asarray(off, np.int64),
        "part_pool": np.asarray(pool, np.uint8),
        **({"chunks": np.asarray(ch, np.int32)} if any(len(r) > 6 for r in rows) else {}),
    }


def mk(costs, cluster, rows, name="adhoc"):
    return Workload(name, costs, cluster, mk_cands(rows))


def stage_costs_uniform(L, pp):
    return [(s * L) // pp for s in range(pp + 1)]
