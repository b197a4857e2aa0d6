"""MI355X-native batched evaluator for DistSim's strategy search (arXiv 2306.08423).

The hot path -- event-flow generation, timeline simulation, strategy search -- lives in
hand-written HIP kernels behind the C ABI of include/distsim.h; `binding` marshals
PyTorch device tensors into those calls.
"""
from .binding import (  # noqa: F401
    Context, DeviceWorkload, DistSimError, Events, SimOutputs, EXPORTS, KERNELS, COL, LIB_PATH,
    alloc_dedup, alloc_events, alloc_events_bound, alloc_outputs, alloc_search, distsim_bubbles, distsim_comm_event_times, distsim_dedup_events, distsim_build_events, distsim_search, distsim_search_static, distsim_simulate, distsim_timeline,
    load_library, stage_entries, stage_rows, upload,
)
