"""Runs a workload through the HIP library (via the C ABI binding) and returns host arrays
shaped like the oracle's, so the two can be compared field by field."""
from __future__ import annotations

import numpy as np
import torch

import paper_2306_08423_amd as ds

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = ds.Context(0)
    return _ctx


_ctx_split = None


def ctx_split():
    """A context whose distsim_simulate gives GPipe candidates their own launch for any list length
    (the default does so from about 10^5 wave-items on)."""
    global _ctx_split
    if _ctx_split is None:
        import os
        old = os.environ.get("DISTSIM_SPLIT_MIN_ITEMS")
        os.environ["DISTSIM_SPLIT_MIN_ITEMS"] = "0"
        try:
            _ctx_split = ds.Context(0)
        finally:
            if old is None:
                del os.environ["DISTSIM_SPLIT_MIN_ITEMS"]
            else:
                os.environ["DISTSIM_SPLIT_MIN_ITEMS"] = old
    return _ctx_split


def run_hip(w, stage_cap=None, util=True, search=None, table=True, split=False):
    """search: None or (objective, weight ndarray or None).  split: through ctx_split()."""
    c = ctx_split() if split else ctx()
    dw = ds.upload(w, c.device)
    cap = ds.stage_entries(w.cand["pp"]) if stage_cap is None else stage_cap
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, cap, table=table)
    # poison the outputs so that untouched entries show up
    ev.status.fill_(-7); ev.stage_pos.fill_(-7); ev.num_events.fill_(-7)
    if table:
        ev.stage_tab.fill_(-7); ev.stage_layers.fill_(-7)
    ds.distsim_build_events(c, dw, ev)
    out = ds.alloc_outputs(c, ev, util=util)
    out.batch_ns.fill_(-7); out.comp_busy_ns.fill_(-7); out.comm_busy_ns.fill_(-7)
    if util:
        out.util.fill_(-7.0)
    ds.distsim_simulate(c, dw.cluster, ev, out)
    res = {}
    if search is not None:
        obj, wgt = search
        best, scratch = ds.alloc_search(c, dw.C)
        wt = torch.from_numpy(np.ascontiguousarray(wgt, dtype=np.int64)).to(c.device) if wgt is not None else None
        ds.distsim_search(c, out.batch_ns, dw.C, best, scratch, weight=wt, objective=obj)
        torch.cuda.synchronize()
        res["best"] = tuple(int(x) for x in best.cpu().numpy())
    torch.cuda.synchronize()
    C = dw.C
    res.update({
        "status": ev.status.cpu().numpy()[:C],
        "num_events": ev.num_events.cpu().numpy()[:C],
        "stage_pos": ev.stage_pos.cpu().numpy()[:C],
        "batch_ns": out.batch_ns.cpu().numpy()[:C],
        "comp_busy_ns": out.comp_busy_ns.cpu().numpy()[:cap],
        "comm_busy_ns": out.comm_busy_ns.cpu().numpy()[:cap],
        "pp": w.cand["pp"].astype(np.int64),
    })
    if util:
        res["util"] = out.util.cpu().numpy()[:cap]
    if table:
        res["stage_tab"] = ev.stage_tab.cpu().numpy()[:, :cap]
        res["stage_layers"] = ev.stage_layers.cpu().numpy()[:cap]
    return res


def rows_of(hip, sel):
    """Per-stage entries of the OK candidates among sel, in sel order."""
    return ds.stage_rows(hip["status"][sel], hip["stage_pos"][sel], hip["pp"][sel])


def assert_same(hip, ora, idx=None, what=""):
    """Bit-exact on every integer output; utilisation (fp64 quotient of two exact integers,
    one IEEE division on both sides) within 1e-12 relative.  idx: the oracle ran on w[idx]."""
    C = len(ora["status"])
    sel = np.arange(C) if idx is None else np.asarray(idx)
    assert np.array_equal(hip["status"][sel], ora["status"]), what + " status"
    assert np.array_equal(hip["batch_ns"][sel], ora["batch_ns"]), what + " batch_ns"
    assert np.array_equal(hip["num_events"][sel], ora["num_events"]), what + " num_events"
    rows, cnt_h = rows_of(hip, sel)
    oo = ora["stage_off"]
    assert np.array_equal(cnt_h, oo[1:] - oo[:-1]), what + " stage counts"
    if len(rows):
        assert rows.min() >= 0 and rows.max() < len(hip["comp_busy_ns"]), what + " stage_pos range"
        assert len(np.unique(rows)) == len(rows), what + " overlapping stage blocks"
    for key in ("comp_busy_ns", "comm_busy_ns"):
        assert np.array_equal(hip[key][rows], ora[key]), what + " " + key
    if "util" in hip:
        a, b = hip["util"][rows], ora["util"]
        assert np.all(np.abs(a - b) <= 1e-12 * np.abs(b)), what + " util"
