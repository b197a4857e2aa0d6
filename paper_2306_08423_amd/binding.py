"""Thin Python binding of the C ABI in include/distsim.h.

Argument marshalling only: every step of the evaluation runs in the HIP kernels of
libdistsim_hip.so.  PyTorch supplies device memory (tensors) and the stream.  There is
no fallback: if the library is missing the import of this module's functions fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistsim_hip.so")

EXPORTS = (
    "distsim_create", "distsim_destroy", "distsim_last_error", "distsim_workspace_bytes", "distsim_stage_entries",
    "distsim_events_bytes", "distsim_events_bind", "distsim_build_events", "distsim_simulate", "distsim_search_scratch_bytes", "distsim_search", "distsim_search_static",
    "distsim_timeline", "distsim_bubbles", "distsim_dedup_workspace_bytes", "distsim_dedup_events", "distsim_comm_event_times",
    "distsim_timing_enable", "distsim_timing_read", "distsim_kernel_name",
)

NCOLS = 8
COL = {"FC": 0, "FA": 1, "BC": 2, "BA": 3, "PF": 4, "PB": 5, "G": 6, "AR": 7}
KERNELS = ("k_layer_tables", "k_decode", "k_bins", "k_scatter", "k_stage_events",
           "k_sim_init", "k_simulate", "k_search", "k_timeline", "k_dedup", "k_comm_event_times", "k_bubbles", "k_simulate_virtual",
           "k_timeline_virtual", "k_simulate_gpipe", "k_simulate_explicit",
           "k_timeline_explicit", "k_compile_schedules", "k_timeline_gpipe")
INT64_MAX = (1 << 63) - 1
ST_OK, ST_INVALID, ST_RANGE, ST_NOROOM, ST_UNSUPPORTED = 0, 1, 2, 3, 4
MAX_PP, MAX_M, MAX_SLOTS = 64, 1 << 16, 2048


class _Costs(C.Structure):
    _fields_ = [("L", C.c_int32), ("V", C.c_int32), ("variant_tp", C.c_void_p),
                ("fwd_comp_ns", C.c_void_p), ("bwd_comp_ns", C.c_void_p),
                ("fwd_comm_ns", C.c_void_p), ("bwd_comm_ns", C.c_void_p),
                ("act_bytes", C.c_void_p), ("grad_bytes", C.c_void_p), ("a2a_bytes", C.c_void_p)]


class _Cluster(C.Structure):
    _fields_ = [("num_devices", C.c_int32), ("gpus_per_node", C.c_int32),
                ("alpha_ns", C.c_int64 * 2), ("beta_bytes_per_ns", C.c_int64 * 2),
                ("dp_bucket_bytes", C.c_int64), ("p2p_blocking", C.c_int32)]


class _Cand(C.Structure):
    _fields_ = [("dp", C.c_void_p), ("tp", C.c_void_p), ("pp", C.c_void_p), ("m", C.c_void_p),
                ("schedule", C.c_void_p), ("part_off", C.c_void_p), ("part_pool", C.c_void_p),
                ("part_pool_len", C.c_int64), ("chunks", C.c_void_p),
                ("n_schedules", C.c_int64), ("schedule_off", C.c_void_p), ("schedule_words", C.c_void_p),
                ("schedule_words_len", C.c_int64)]


class _Events(C.Structure):
    _fields_ = [("stage_cap", C.c_int64), ("L", C.c_int32), ("V", C.c_int32),
                ("status", C.c_void_p), ("stage_pos", C.c_void_p), ("stage_tab", C.c_void_p),
                ("stage_layers", C.c_void_p), ("num_events", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("num_candidates", C.c_int64)]


_lib = None


def load_library():
    """dlopen the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with paper_2306_08423_amd.build.build_library()")
    lib = C.CDLL(LIB_PATH)
    lib.distsim_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
    lib.distsim_create.restype = C.c_int
    lib.distsim_destroy.argtypes = [C.c_void_p]
    lib.distsim_destroy.restype = None
    lib.distsim_last_error.argtypes = [C.c_void_p]
    lib.distsim_last_error.restype = C.c_char_p
    lib.distsim_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int64]
    lib.distsim_workspace_bytes.restype = C.c_size_t
    lib.distsim_stage_entries.argtypes = [C.c_int64]
    lib.distsim_stage_entries.restype = C.c_int64
    lib.distsim_build_events.argtypes = [C.c_void_p, C.POINTER(_Costs), C.POINTER(_Cluster), C.POINTER(_Cand),
                                         C.c_int64, C.POINTER(_Events), C.c_void_p]
    lib.distsim_build_events.restype = C.c_int
    lib.distsim_events_bytes.argtypes = [C.POINTER(_Costs), C.c_int64, C.c_int64, C.c_int]
    lib.distsim_events_bytes.restype = C.c_size_t
    lib.distsim_events_bind.argtypes = [C.POINTER(_Events), C.c_void_p, C.c_size_t, C.POINTER(_Costs), C.c_int64,
                                        C.c_int64, C.c_int]
    lib.distsim_events_bind.restype = C.c_int
    lib.distsim_simulate.argtypes = [C.c_void_p, C.POINTER(_Cluster), C.POINTER(_Cand), C.POINTER(_Events), C.c_int64,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.distsim_simulate.restype = C.c_int
    lib.distsim_search_scratch_bytes.argtypes = [C.c_int64]
    lib.distsim_search_scratch_bytes.restype = C.c_size_t
    lib.distsim_search.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p,
                                   C.c_void_p, C.c_void_p]
    lib.distsim_search.restype = C.c_int
    lib.distsim_search_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
    lib.distsim_search_static.restype = C.c_int
    lib.distsim_timeline.argtypes = [C.c_void_p, C.POINTER(_Cluster), C.POINTER(_Cand), C.POINTER(_Events), C.c_int64] + [C.c_void_p] * 7
    lib.distsim_timeline.restype = C.c_int
    lib.distsim_bubbles.argtypes = [C.c_void_p, C.POINTER(_Cand), C.POINTER(_Events), C.c_int64] + [C.c_void_p] * 6
    lib.distsim_bubbles.restype = C.c_int
    lib.distsim_dedup_workspace_bytes.argtypes = [C.c_int64]
    lib.distsim_dedup_workspace_bytes.restype = C.c_size_t
    lib.distsim_dedup_events.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.distsim_dedup_events.restype = C.c_int
    lib.distsim_comm_event_times.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 6
    lib.distsim_comm_event_times.restype = C.c_int
    lib.distsim_timing_enable.argtypes = [C.c_void_p, C.c_int]
    lib.distsim_timing_enable.restype = C.c_int
    lib.distsim_timing_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.distsim_timing_read.restype = C.c_int
    lib.distsim_kernel_name.argtypes = [C.c_int]
    lib.distsim_kernel_name.restype = C.c_char_p
    _lib = lib
    return lib


class DistSimError(RuntimeError):
    pass


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """distsim_ctx bound to one HIP device."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        h = C.c_void_p()
        rc = self.lib.distsim_create(C.byref(h), device)
        if rc != 0:
            raise DistSimError(f"distsim_create failed ({rc})")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.distsim_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc: int):
        if rc != 0:
            raise DistSimError(f"distsim error {rc}: {self.lib.distsim_last_error(self.h).decode()}")

    def timing_enable(self, on: bool = True):
        self.check(self.lib.distsim_timing_enable(self.h, int(on)))

    def timing_read(self) -> Dict[str, tuple]:
        out = {}
        for k, name in enumerate(KERNELS):
            ms, n = C.c_double(), C.c_int64()
            self.check(self.lib.distsim_timing_read(self.h, k, C.byref(ms), C.byref(n)))
            out[name] = (ms.value, n.value)
        return out


@dataclass
class DeviceWorkload:
    """Device-resident copy of a cost table, a cluster and a candidate list."""
    L: int
    V: int
    C: int
    costs: Dict[str, torch.Tensor]
    cluster: Dict[str, object]
    cand: Dict[str, torch.Tensor]

    def costs_struct(self) -> _Costs:
        c = self.costs
        return _Costs(self.L, self.V, _ptr(c["variant_tp"]), _ptr(c["fwd_comp_ns"]), _ptr(c["bwd_comp_ns"]),
                      _ptr(c["fwd_comm_ns"]), _ptr(c["bwd_comm_ns"]), _ptr(c["act_bytes"]), _ptr(c["grad_bytes"]),
                      _ptr(c.get("a2a_bytes")))

    def cluster_struct(self) -> _Cluster:
        return cluster_struct(self.cluster)

    def cand_struct(self) -> _Cand:
        k = self.cand
        pool = k["part_pool"]
        soff, swords = k.get("schedule_off"), k.get("schedule_words")
        nsched = int(soff.numel()) - 1 if soff is not None and swords is not None and swords.numel() else 0
        return _Cand(_ptr(k["dp"]), _ptr(k["tp"]), _ptr(k["pp"]), _ptr(k["m"]), _ptr(k["schedule"]),
                     _ptr(k["part_off"]), _ptr(pool) if pool.numel() else None, pool.numel(), _ptr(k.get("chunks")),
                     max(nsched, 0), _ptr(soff) if nsched > 0 else None, _ptr(swords) if nsched > 0 else None,
                     int(swords.numel()) if nsched > 0 else 0)


def cluster_struct(cl) -> _Cluster:
    return _Cluster(int(cl["num_devices"]), int(cl["gpus_per_node"]),
                    (C.c_int64 * 2)(*[int(x) for x in cl["alpha_ns"]]),
                    (C.c_int64 * 2)(*[int(x) for x in cl["beta_bytes_per_ns"]]),
                    int(cl["dp_bucket_bytes"]), int(cl.get("p2p_blocking", 0)))


def upload(w, device) -> DeviceWorkload:
    """Copy a workloads.Workload (numpy, host) to the device, unchanged."""
    dev = torch.device(device)
    co = {k: torch.from_numpy(v).contiguous().to(dev) for k, v in w.costs.items() if hasattr(v, "dtype")}
    ca = {k: torch.from_numpy(v).contiguous().to(dev) for k, v in w.cand.items()}
    return DeviceWorkload(int(w.costs["L"]), int(w.costs["V"]), int(w.cand["dp"].shape[0]), co, dict(w.cluster), ca)


@dataclass
class Events:
    """Caller-owned device buffers of a distsim_events plus the ctypes view of them."""
    C: int
    stage_cap: int
    status: torch.Tensor
    stage_pos: torch.Tensor
    stage_tab: Optional[torch.Tensor]
    stage_layers: Optional[torch.Tensor]
    num_events: torch.Tensor
    workspace: torch.Tensor
    struct: _Events


def stage_entries(pp) -> int:
    """Tight stage_cap for a host-side array of stage counts: every candidate takes pp rounded
    up to a power of two, candidates of one size class are packed 64 entries to a wavefront."""
    import numpy as np
    pp = np.clip(np.asarray(pp, dtype=np.int64), 1, 64)
    width = 1 << np.ceil(np.log2(pp)).astype(np.int64)
    total = 0
    for k in range(7):
        n = int((width == (64 >> k)).sum())
        total += -(-n // (1 << k)) * 64
    return total


def stage_rows(status, stage_pos, pp):
    """Host-side index helper: positions in the per-stage arrays of the stages of every OK
    candidate, concatenated in candidate order, and the per-candidate counts."""
    import numpy as np
    ok = np.asarray(status) == 0
    cnt = np.where(ok, np.asarray(pp, dtype=np.int64), 0)
    start = np.where(ok, np.asarray(stage_pos, dtype=np.int64), 0)
    first = np.repeat(np.cumsum(cnt) - cnt, cnt)
    return np.repeat(start, cnt) + (np.arange(int(cnt.sum())) - first), cnt


def alloc_events(ctx: Context, L: int, V: int, Cn: int, stage_cap: Optional[int] = None,
                 table: bool = True) -> Events:
    """table=False: no stage table is written (distsim_simulate composes the stage events itself)."""
    dev = ctx.device
    if stage_cap is None:
        stage_cap = ctx.lib.distsim_stage_entries(Cn)
    nbytes = ctx.lib.distsim_workspace_bytes(L, V, Cn)
    if nbytes == 0:
        raise DistSimError("distsim_workspace_bytes rejected (L, V, C)")
    status = torch.empty(max(Cn, 1), dtype=torch.int32, device=dev)
    stage_pos = torch.empty(max(Cn, 1), dtype=torch.int64, device=dev)
    cap = max(int(stage_cap), 0)
    stage_tab = torch.empty((NCOLS, max(cap, 1)), dtype=torch.int64, device=dev) if table else None
    stage_layers = torch.empty(max(cap, 1), dtype=torch.int32, device=dev) if table else None
    num_events = torch.empty(max(Cn, 1), dtype=torch.int64, device=dev)
    # torch's caching allocator hands out 512-byte aligned blocks
    workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    st = _Events(cap, 0, 0, _ptr(status), _ptr(stage_pos), _ptr(stage_tab), _ptr(stage_layers), _ptr(num_events),
                 _ptr(workspace), nbytes, 0)
    return Events(Cn, cap, status, stage_pos, stage_tab, stage_layers, num_events, workspace, st)


def alloc_events_bound(ctx: Context, dw: DeviceWorkload, stage_cap: int, table: bool = True) -> Events:
    """The same arrays carved out of ONE device allocation by distsim_events_bind."""
    co = dw.costs_struct()
    nbytes = ctx.lib.distsim_events_bytes(C.byref(co), dw.C, int(stage_cap), int(table))
    if nbytes == 0:
        raise DistSimError("distsim_events_bytes rejected its arguments")
    blob = torch.empty(nbytes, dtype=torch.uint8, device=ctx.device)
    st = _Events()
    rc = ctx.lib.distsim_events_bind(C.byref(st), _ptr(blob), nbytes, C.byref(co), dw.C, int(stage_cap), int(table))
    if rc != 0:
        raise DistSimError(f"distsim_events_bind failed ({rc})")
    base = blob.data_ptr()

    def view(ptr, n, dtype, shape=None):
        if not ptr:
            return None
        size = torch.empty(0, dtype=dtype).element_size()
        t = blob[ptr - base: ptr - base + n * size].view(dtype)
        return t if shape is None else t.view(shape)
    Cn, cap = max(dw.C, 1), max(int(stage_cap), 1)
    return Events(dw.C, int(stage_cap), view(st.status, Cn, torch.int32), view(st.stage_pos, Cn, torch.int64),
                  view(st.stage_tab, NCOLS * cap, torch.int64, (NCOLS, cap)), view(st.stage_layers, cap, torch.int32),
                  view(st.num_events, Cn, torch.int64), blob, st)


def distsim_build_events(ctx: Context, dw: DeviceWorkload, ev: Events) -> None:
    co, cl, ca = dw.costs_struct(), dw.cluster_struct(), dw.cand_struct()
    ctx.check(ctx.lib.distsim_build_events(ctx.h, C.byref(co), C.byref(cl), C.byref(ca), dw.C, C.byref(ev.struct),
                                           _stream()))


@dataclass
class SimOutputs:
    batch_ns: torch.Tensor
    comp_busy_ns: torch.Tensor
    comm_busy_ns: torch.Tensor
    util: Optional[torch.Tensor]


def alloc_outputs(ctx: Context, ev: Events, util: bool = True) -> SimOutputs:
    dev = ctx.device
    n = max(ev.stage_cap, 1)
    return SimOutputs(torch.empty(max(ev.C, 1), dtype=torch.int64, device=dev),
                      torch.empty(n, dtype=torch.int64, device=dev),
                      torch.empty(n, dtype=torch.int64, device=dev),
                      torch.empty(n, dtype=torch.float64, device=dev) if util else None)


def distsim_simulate(ctx: Context, dw: DeviceWorkload, ev: Events, out: SimOutputs) -> None:
    cl, ca = dw.cluster_struct(), dw.cand_struct()
    ctx.check(ctx.lib.distsim_simulate(ctx.h, C.byref(cl), C.byref(ca), C.byref(ev.struct), ev.C, _ptr(out.batch_ns),
                                       _ptr(out.comp_busy_ns), _ptr(out.comm_busy_ns), _ptr(out.util), _stream()))


def alloc_search(ctx: Context, Cn: int):
    n = ctx.lib.distsim_search_scratch_bytes(Cn)
    return (torch.empty(2, dtype=torch.int64, device=ctx.device),
            torch.empty(max(n, 8), dtype=torch.uint8, device=ctx.device))


def distsim_search(ctx: Context, batch_ns: torch.Tensor, Cn: int, best: torch.Tensor, scratch: torch.Tensor,
                   weight: Optional[torch.Tensor] = None, objective: int = 0) -> None:
    ctx.check(ctx.lib.distsim_search(ctx.h, _ptr(batch_ns), _ptr(weight), Cn, objective, _ptr(best), _ptr(scratch),
                                     _stream()))


def distsim_search_static(ctx: Context, batch_ns: torch.Tensor, Cn: int, best: torch.Tensor,
                          weight: Optional[torch.Tensor] = None, objective: int = 0) -> None:
    """distsim_search with the partial results in the library's own device array: no scratch argument."""
    ctx.check(ctx.lib.distsim_search_static(ctx.h, _ptr(batch_ns), _ptr(weight), Cn, objective, _ptr(best), _stream()))


def distsim_timeline(ctx: Context, dw: DeviceWorkload, ev: Events, sel: torch.Tensor, task_off: torch.Tensor,
                     start_ns: torch.Tensor, end_ns: torch.Tensor, ar_start_ns: torch.Tensor,
                     ar_end_ns: torch.Tensor) -> None:
    cl, ca = dw.cluster_struct(), dw.cand_struct()
    ctx.check(ctx.lib.distsim_timeline(ctx.h, C.byref(cl), C.byref(ca), C.byref(ev.struct), sel.numel(), _ptr(sel), _ptr(task_off),
                                       _ptr(start_ns), _ptr(end_ns), _ptr(ar_start_ns), _ptr(ar_end_ns), _stream()))


def distsim_bubbles(ctx: Context, dw: DeviceWorkload, ev: Events, sel: torch.Tensor, task_off: torch.Tensor,
                    start_ns: torch.Tensor, end_ns: torch.Tensor, idle_before_ns: torch.Tensor) -> None:
    ca = dw.cand_struct()
    ctx.check(ctx.lib.distsim_bubbles(ctx.h, C.byref(ca), C.byref(ev.struct), sel.numel(), _ptr(sel), _ptr(task_off),
                                      _ptr(start_ns), _ptr(end_ns), _ptr(idle_before_ns), _stream()))


def distsim_dedup_events(ctx: Context, records: torch.Tensor, event_id: torch.Tensor, rep: torch.Tensor,
                         num_events: torch.Tensor, workspace: torch.Tensor) -> None:
    """records [n][K] int64; event_id, rep [n] int32; num_events [1] int64; workspace uint8."""
    n, K = (int(records.shape[0]), int(records.shape[1])) if records.dim() == 2 else (0, 1)
    ctx.check(ctx.lib.distsim_dedup_events(ctx.h, _ptr(records), n, K, _ptr(event_id), _ptr(rep), _ptr(num_events),
                                           _ptr(workspace), workspace.numel(), _stream()))


def distsim_comm_event_times(ctx: Context, kind: torch.Tensor, ranks: torch.Tensor, t_a: torch.Tensor,
                             t_b: torch.Tensor, elapsed_ns: torch.Tensor) -> None:
    ctx.check(ctx.lib.distsim_comm_event_times(ctx.h, kind.numel(), _ptr(kind), _ptr(ranks), _ptr(t_a), _ptr(t_b),
                                               _ptr(elapsed_ns), _stream()))


def alloc_dedup(ctx: Context, n: int, device) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """event_id, rep, num_events and the workspace for distsim_dedup_events on n records."""
    nbytes = int(ctx.lib.distsim_dedup_workspace_bytes(n))
    return (torch.empty(max(n, 1), dtype=torch.int32, device=device),
            torch.full((max(n, 1),), -1, dtype=torch.int32, device=device),
            torch.zeros(1, dtype=torch.int64, device=device),
            torch.empty(max(nbytes, 1), dtype=torch.uint8, device=device))
