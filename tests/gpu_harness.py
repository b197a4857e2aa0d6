"""Runs a workload through the HIP library (via the C ABI binding) and returns host arrays
shaped like the oracle's, so the two can be compared field by field."""
from __future__ import annotations

import numpy as np
import torch

import paper_2306_08423_amd as ds
from workloads import total_stages

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = ds.Context(0)
    return _ctx


def run_hip(w, stage_cap=None, util=True, search=None):
    """search: None or (objective, weight ndarray or None)."""
    c = ctx()
    dw = ds.upload(w, c.device)
    cap = total_stages(w) if stage_cap is None else stage_cap
    ev = ds.alloc_events(c, dw.L, dw.V, dw.C, cap)
    # poison the outputs so that untouched entries show up
    ev.status.fill_(-7); ev.stage_off.fill_(-7); ev.num_events.fill_(-7)
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
    soff = ev.stage_off.cpu().numpy()
    n = int(soff[C])
    res.update({
        "status": ev.status.cpu().numpy()[:C],
        "num_events": ev.num_events.cpu().numpy()[:C],
        "stage_off": soff,
        "stage_tab": ev.stage_tab.cpu().numpy()[:, :min(n, cap)],
        "stage_layers": ev.stage_layers.cpu().numpy()[:min(n, cap)],
        "batch_ns": out.batch_ns.cpu().numpy()[:C],
        "comp_busy_ns": out.comp_busy_ns.cpu().numpy()[:min(n, cap)],
        "comm_busy_ns": out.comm_busy_ns.cpu().numpy()[:min(n, cap)],
    })
    if util:
        res["util"] = out.util.cpu().numpy()[:min(n, cap)]
    return res


def assert_same(hip, ora, idx=None, what=""):
    """Bit-exact on every integer output; utilisation (fp64 quotient of two exact integers,
    one IEEE division on both sides) within 1e-12 relative.  idx: the oracle ran on w[idx]."""
    C = len(ora["status"])
    sel = np.arange(C) if idx is None else np.asarray(idx)
    assert np.array_equal(hip["status"][sel], ora["status"]), what + " status"
    assert np.array_equal(hip["batch_ns"][sel], ora["batch_ns"]), what + " batch_ns"
    assert np.array_equal(hip["num_events"][sel], ora["num_events"]), what + " num_events"
    ho, oo = hip["stage_off"], ora["stage_off"]
    cnt_h = (ho[1:] - ho[:-1])[sel]
    cnt_o = oo[1:] - oo[:-1]
    assert np.array_equal(cnt_h, cnt_o), what + " stage counts"
    if idx is None:
        assert np.array_equal(ho, oo), what + " stage_off"
    # gather the ragged rows of the selected candidates
    starts = ho[:-1][sel]
    rows = np.repeat(starts, cnt_o) + (np.arange(int(cnt_o.sum())) - np.repeat(oo[:-1], cnt_o))
    for key in ("comp_busy_ns", "comm_busy_ns"):
        assert np.array_equal(hip[key][rows], ora[key]), what + " " + key
    if "util" in hip:
        a, b = hip["util"][rows], ora["util"]
        assert np.all(np.abs(a - b) <= 1e-12 * np.abs(b)), what + " util"
