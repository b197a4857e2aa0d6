"""Oracle for the bubble analysis of a dumped timeline.  TEST INFRASTRUCTURE ONLY (tests/, smoke,
the benchmark's CPU leg).

The timeline says at what time which device computes or communicates, and the paper lists bubble
analysis among its uses next to iteration time and utilisation (Sec. 3.2); the per-stage,
per-micro-batch timestamps are what a user finds the bubbles with (Sec. 5).  A bubble is
the idle time of a device in front of a stage-task: start of the task minus end of the task the
device ran before it (minus 0, the start of the iteration, for its first task).  The device order is
written out here as explicit lists, the way the schedule defines it (Sec. 2.1.3, Fig. 2: GPipe =
all forwards then all backwards; Dapple = warm-up forwards, one-forward-one-backward, cool-down).
"""
import numpy as np


def device_order(pp: int, m: int, schedule: int, s: int):
    """[(kind, micro-batch)] in the order device s runs its stage-tasks; kind 0 = forward."""
    if schedule == 0:
        return [(0, j) for j in range(m)] + [(1, j) for j in range(m)]
    w = min(pp - 1 - s, m)
    order = [(0, j) for j in range(w)]
    f, b = w, 0
    while f < m:
        order.append((0, f)); f += 1
        order.append((1, b)); b += 1
    while b < m:
        order.append((1, b)); b += 1
    return order


def idle_before(start: np.ndarray, end: np.ndarray, schedule: int) -> np.ndarray:
    """start, end [2][pp][m] of one candidate -> idle time in front of every stage-task, same shape."""
    _, pp, m = start.shape
    out = np.zeros_like(start)
    for s in range(pp):
        prev_end = 0
        for kind, j in device_order(pp, m, schedule, s):
            out[kind, s, j] = int(start[kind, s, j]) - prev_end
            prev_end = int(end[kind, s, j])
    return out
