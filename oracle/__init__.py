"""ctypes front end of the CPU oracle (``distsim_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Imported by ``tests/``, by the smoke check and by the benchmark's CPU-baseline
leg; never by the product package.  It knows nothing about the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "distsim_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

INT64_MAX = np.iinfo(np.int64).max


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a checker being built is not the checker being used)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_simulate.restype = ctypes.c_int
        _lib.oracle_search.restype = ctypes.c_int
        _lib.oracle_stage_table.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def simulate(w, nthreads: int = 1, timeline: bool = False) -> Dict[str, np.ndarray]:
    """Evaluate every candidate of workload ``w``.

    Returns status[C], batch_ns[C], num_events[C], stage_off[C+1] and the ragged
    per-stage arrays comp_busy_ns / comm_busy_ns / util (index stage_off[c] + s).
    ``timeline=True`` (single candidate only) adds start/end[2][pp][m] of every
    forward (0) and backward (1) stage-task and ar_window[2][pp]: start of the first and
    end of the last gradient all-reduce event of every stage (-1 = none).
    """
    lib = _load()
    co, cl, ca = w.costs, w.cluster, w.cand
    L, V = int(co["L"]), int(co["V"])
    vt = _c(co["variant_tp"], np.int32)
    cols = [_c(co[k], np.int64) for k in
            ("fwd_comp_ns", "bwd_comp_ns", "fwd_comm_ns", "bwd_comm_ns", "act_bytes", "grad_bytes", "a2a_bytes")]
    for a in cols:
        assert a.size == V * L
    alpha = _c(cl["alpha_ns"], np.int64)
    beta = _c(cl["beta_bytes_per_ns"], np.int64)
    dp, tp, pp, m = (_c(ca[k], np.int32) for k in ("dp", "tp", "pp", "m"))
    sched = _c(ca["schedule"], np.uint8)
    chunks = _c(ca["chunks"], np.int32) if ca.get("chunks") is not None else None
    poff = _c(ca["part_off"], np.int64)
    pool = _c(ca["part_pool"], np.uint8)
    # explicit schedules (schedule 4): offsets [n+1] and the word pool; a candidate names its schedule in "chunks"
    xoff = _c(ca["schedule_off"], np.int64) if ca.get("schedule_off") is not None else None
    xwords = _c(ca["schedule_words"], np.int32) if ca.get("schedule_words") is not None else None
    xn = (xoff.shape[0] - 1) if xoff is not None else 0
    xlen = int(xwords.size) if xwords is not None else 0
    if xwords is not None and xwords.size == 0:
        xwords = np.zeros(1, np.int32)
    pool_len = int(pool.size)
    if pool.size == 0:
        pool = np.zeros(1, np.uint8)
    C = dp.shape[0]
    S = int(np.clip(pp.astype(np.int64), 0, None).sum())
    status = np.empty(C, np.int32)
    batch = np.empty(C, np.int64)
    nev = np.empty(C, np.int64)
    soff = np.empty(C + 1, np.int64)
    comp = np.zeros(max(S, 1), np.int64)
    comm = np.zeros(max(S, 1), np.int64)
    util = np.zeros(max(S, 1), np.float64)
    tls = tle = tar = None
    if timeline:
        assert C == 1
        rows = int(pp[0]) * (int(chunks[0]) if chunks is not None and sched[0] == 3 else 1)   # virtual stages
        if sched[0] == 4 and chunks is not None and xoff is not None and 0 <= int(chunks[0]) < xn:
            o = int(xoff[int(chunks[0])])
            if 0 <= o and o + 5 <= xlen:
                rows = max(1, int(xwords[o + 1]))     # S of its schedule block
        tls = np.full((2, rows, int(m[0])), -1, np.int64)
        tle = np.full((2, rows, int(m[0])), -1, np.int64)
        tar = np.full((2, int(pp[0])), -1, np.int64)
    rc = lib.oracle_simulate(
        ctypes.c_int32(L), ctypes.c_int32(V), _p(vt), *[_p(a) for a in cols],
        ctypes.c_int32(int(cl["num_devices"])), ctypes.c_int32(int(cl["gpus_per_node"])),
        _p(alpha), _p(beta), ctypes.c_int64(int(cl["dp_bucket_bytes"])), ctypes.c_int32(int(cl.get("p2p_blocking", 0))),
        ctypes.c_int64(C), _p(dp), _p(tp), _p(pp), _p(m), _p(sched), _p(chunks), _p(poff), _p(pool), ctypes.c_int64(pool_len),
        ctypes.c_int64(xn), _p(xoff), _p(xwords), ctypes.c_int64(xlen),
        _p(status), _p(batch), _p(nev), _p(soff), _p(comp), _p(comm), _p(util),
        _p(tls), _p(tle), _p(tar), ctypes.c_int32(int(nthreads)))
    if rc != 0:
        raise ValueError(f"oracle_simulate rejected its arguments (rc={rc})")
    n = int(soff[C])
    out = {"status": status, "batch_ns": batch, "num_events": nev, "stage_off": soff,
           "comp_busy_ns": comp[:n], "comm_busy_ns": comm[:n], "util": util[:n]}
    if timeline:
        out["start"], out["end"], out["ar_window"] = tls, tle, tar
    return out


def search(batch_ns, weight=None, objective: int = 0):
    """Return (best_index or -1, batch_ns of it)."""
    lib = _load()
    b = _c(batch_ns, np.int64)
    wt = _c(weight, np.int64) if weight is not None else None
    if objective == 1:
        assert wt is not None and wt.shape == b.shape
    best = np.zeros(2, np.int64)
    lib.oracle_search(_p(b), _p(wt), ctypes.c_int64(b.shape[0]), ctypes.c_int32(objective), _p(best))
    return int(best[0]), int(best[1])


def stage_table(w, sim) -> Dict[str, np.ndarray]:
    """The composed events of every stage of the candidates that ``sim`` (a result of ``simulate`` on
    the same workload) reports as OK, from plain loops over each stage's layers: ``tab`` [8][n] with
    the columns FC, FA, BC, BA, PF, PB, G, AR and ``layer_lo`` / ``layer_hi`` [n], n = stage_off[C],
    entry stage_off[c] + s.  Candidates of the schedules 3 and 4 keep zeros."""
    lib = _load()
    co, cl, ca = w.costs, w.cluster, w.cand
    L, V = int(co["L"]), int(co["V"])
    vt = _c(co["variant_tp"], np.int32)
    cols = [_c(co[k], np.int64) for k in
            ("fwd_comp_ns", "bwd_comp_ns", "fwd_comm_ns", "bwd_comm_ns", "act_bytes", "grad_bytes", "a2a_bytes")]
    alpha = _c(cl["alpha_ns"], np.int64)
    beta = _c(cl["beta_bytes_per_ns"], np.int64)
    dp, tp, pp = (_c(ca[k], np.int32) for k in ("dp", "tp", "pp"))
    sched = _c(ca["schedule"], np.uint8)
    poff = _c(ca["part_off"], np.int64)
    pool = _c(ca["part_pool"], np.uint8)
    if pool.size == 0:
        pool = np.zeros(1, np.uint8)
    C = dp.shape[0]
    status = _c(sim["status"], np.int32)
    soff = _c(sim["stage_off"], np.int64)
    n = int(soff[C])
    tab = np.zeros((8, max(n, 1)), np.int64)
    lo = np.zeros(max(n, 1), np.int32)
    hi = np.zeros(max(n, 1), np.int32)
    rc = lib.oracle_stage_table(
        ctypes.c_int32(L), ctypes.c_int32(V), _p(vt), *[_p(a) for a in cols],
        ctypes.c_int32(int(cl["num_devices"])), ctypes.c_int32(int(cl["gpus_per_node"])), _p(alpha), _p(beta),
        ctypes.c_int64(C), _p(dp), _p(tp), _p(pp), _p(sched), _p(poff), _p(pool), _p(status), _p(soff),
        _p(tab), _p(lo), _p(hi))
    if rc != 0:
        raise ValueError(f"oracle_stage_table rejected its arguments (rc={rc})")
    if n == 0:
        return {"tab": tab[:, :0], "layer_lo": lo[:0], "layer_hi": hi[:0]}
    return {"tab": tab, "layer_lo": lo, "layer_hi": hi}
