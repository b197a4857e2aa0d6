"""Oracle for the two steps in front of event-flow generation.  TEST INFRASTRUCTURE ONLY:
imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg, never by the
product path.

* dedup_events  -- Sec. 4.1 (event generator): operators with the same name, parameters and
  input shape (and intra-/inter-node attribute) are one event.  Written as the definition: walk
  the operators in order and keep a dictionary of the ones seen.
* comm_event_times -- Sec. 4.2 (profiling events): a point-to-point event lasts the minimum of
  the SEND and the RECV call; an all-reduce over N > 8 devices is the 8-device profile scaled by
  the ratio of the ring volumes 2(N-1)P/N, i.e. by 8(N-1)/(7N).  Exact integers (Python ints),
  truncated.
"""
from typing import Tuple

import numpy as np


def dedup_events(records: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """records [n][K] int64 -> (event_id [n] int32, rep [num_events] int32): events numbered in
    the order of their first operator, rep[e] = index of that operator."""
    records = np.asarray(records, dtype=np.int64)
    n = records.shape[0]
    event_id = np.empty(n, dtype=np.int32)
    seen = {}
    rep = []
    for i in range(n):
        key = records[i].tobytes()
        e = seen.get(key)
        if e is None:
            e = len(rep)
            seen[key] = e
            rep.append(i)
        event_id[i] = e
    return event_id, np.asarray(rep, dtype=np.int32)


def comm_event_times(kind, ranks, t_a, t_b) -> np.ndarray:
    """Elapsed ns of each communication event; -1 for a record that is not one."""
    out = np.empty(len(kind), dtype=np.int64)
    for i, (kd, N, a, b) in enumerate(zip(kind.tolist(), ranks.tolist(), t_a.tolist(), t_b.tolist())):
        e = -1
        if kd == 0:
            if a >= 0 and b >= 0:
                e = min(a, b)
        elif kd == 1 and N >= 1 and a >= 0:
            e = a if N <= 8 else (a * 8 * (N - 1)) // (7 * N)
        out[i] = e
    return out
