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
    ds.distsim_simulate(c, dw, ev, out)
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
        "workload": w,
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


def beyond_limits(w):
    """Per candidate: does it lie beyond what this library's kernels take (include/distsim.h,
    DISTSIM_ST_UNSUPPORTED)?  From the inputs alone; says nothing about validity."""
    ca = w.cand
    C = len(ca["pp"])
    pp, m, sc = ca["pp"].astype(np.int64), ca["m"].astype(np.int64), ca["schedule"]
    out = m > ds.binding.MAX_M
    ch = ca.get("chunks")
    if ch is not None:
        ch = ch.astype(np.int64)
        out = out | ((sc == 3) & (pp * ch > ds.binding.MAX_PP))
        off, words = ca.get("schedule_off"), ca.get("schedule_words")
        if off is not None and words is not None:
            n = len(off) - 1
            for c in np.nonzero(sc == 4)[0]:
                sid = int(ch[c])
                if not (0 <= sid < n):
                    continue
                o, e = int(off[sid]), int(off[sid + 1])
                if o < 0 or e - o < 5 or e > len(words):
                    continue
                S, nparts = int(words[o + 1]), int(words[o + 3])
                if S > ds.binding.MAX_PP or nparts > ds.binding.MAX_PP or S * int(m[c]) > ds.binding.MAX_SLOTS:
                    out[c] = True
    return out


def assert_same(hip, ora, idx=None, what="", w=None):
    """Bit-exact on every integer output; utilisation (fp64 quotient of two exact integers,
    one IEEE division on both sides) within 1e-12 relative.  idx: the oracle ran on w[idx].
    w: the workload (default: the one run_hip was given).  Candidates of it that lie beyond the
    library's limits must come back as DISTSIM_ST_UNSUPPORTED (unless they fail an O(1) validity check, which both
    sides report as invalid) and are left out of the comparison of results; no other candidate may."""
    C = len(ora["status"])
    sel = np.arange(C) if idx is None else np.asarray(idx)
    w = hip.get("workload") if w is None else w
    hs, os_ = hip["status"][sel], ora["status"]
    unsup = hs == ds.binding.ST_UNSUPPORTED
    if w is None:
        assert not unsup.any(), what + " unsupported candidates in a workload within the limits"
    else:
        beyond = beyond_limits(w)[sel]
        assert not (unsup & ~beyond).any(), what + " unsupported without a limit being passed"
        assert np.isin(hs[beyond], (ds.binding.ST_INVALID, ds.binding.ST_UNSUPPORTED)).all(), what + " beyond the limits but simulated"
        assert (hs[beyond & (os_ != 1)] == ds.binding.ST_UNSUPPORTED).all(), what + " valid beyond the limits, not reported as such"
        assert (hip["batch_ns"][sel][unsup] == np.iinfo(np.int64).max).all() and (hip["num_events"][sel][unsup] == 0).all()
        assert (hip["stage_pos"][sel][unsup] == -1).all()
    keep = ~unsup
    assert np.array_equal(hs[keep], os_[keep]), what + " status"
    assert np.array_equal(hip["batch_ns"][sel][keep], ora["batch_ns"][keep]), what + " batch_ns"
    assert np.array_equal(hip["num_events"][sel][keep], ora["num_events"][keep]), what + " num_events"
    rows, cnt_h = rows_of(hip, sel)
    oo = ora["stage_off"]
    cnt_o = (oo[1:] - oo[:-1]) * keep                       # the oracle's rows of the candidates the library took
    assert np.array_equal(cnt_h, cnt_o), what + " stage counts"
    orow = np.repeat(oo[:-1], cnt_o) + (np.arange(int(cnt_o.sum())) - np.repeat(np.cumsum(cnt_o) - cnt_o, cnt_o))
    if len(rows):
        assert rows.min() >= 0 and rows.max() < len(hip["comp_busy_ns"]), what + " stage_pos range"
        assert len(np.unique(rows)) == len(rows), what + " overlapping stage blocks"
    for key in ("comp_busy_ns", "comm_busy_ns"):
        assert np.array_equal(hip[key][rows], ora[key][orow]), what + " " + key
    if "util" in hip:
        a, b = hip["util"][rows], ora["util"][orow]
        assert np.all(np.abs(a - b) <= 1e-12 * np.abs(b)), what + " util"
    if "stage_tab" in hip and "stage_table" in ora:
        # every column of the materialised stage table and the layer ranges, against the per-stage
        # sums that the oracle forms with plain loops over each stage's layers
        t = ora["stage_table"]
        names = ("FC", "FA", "BC", "BA", "PF", "PB", "G", "AR")
        for col, nm in enumerate(names):
            assert np.array_equal(hip["stage_tab"][col, rows], t["tab"][col, orow]), what + " stage_tab " + nm
        lay = hip["stage_layers"][rows]
        assert np.array_equal(lay & 0xff, t["layer_lo"][orow]) and np.array_equal(lay >> 8, t["layer_hi"][orow]), what + " stage_layers"
        # entries of the rows in use that belong to no candidate are zero (whole lists only)
        used = (int(rows.max()) // 64 + 1) * 64 if len(rows) and idx is None else 0
        free = np.ones(used, bool)
        free[rows[rows < used]] = False
        assert not hip["stage_tab"][:, :used][:, free].any() and not hip["stage_layers"][:used][free].any(), what + " free rows"


def oracle_with_table(oracle_mod, w, nthreads=1):
    """The oracle's results plus its stage table (the yardstick of stage_tab / stage_layers)."""
    ora = oracle_mod.simulate(w, nthreads=nthreads)
    ora["stage_table"] = oracle_mod.stage_table(w, ora)
    return ora
