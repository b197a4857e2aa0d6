"""Oracle for the bubble analysis of a dumped timeline.  TEST INFRASTRUCTURE ONLY (tests/, smoke,
the benchmark's CPU leg).

The timeline says at what time which device computes or communicates, and the paper lists bubble
analysis among its uses next to iteration time and utilisation (Sec. 3.2); the per-stage,
per-micro-batch timestamps are what a user finds the bubbles with (Sec. 5).  A bubble is
the idle time of a device in front of a stage-task: start of the task minus end of the task the
device ran before it (minus 0, the start of the iteration, for its first task).  The device order is
written out here as explicit lists, the way the schedule defines it (Sec. 2.1.3, Fig. 2: GPipe =
all forwards then all backwards; Dapple = warm-up forwards, one-forward-one-backward, cool-down;
the interleaved variant runs the same pattern over (chunk, micro-batch) slots).
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


def device_order_interleaved(pp: int, m: int, chunks: int, d: int):
    """[(kind, virtual stage, micro-batch)] in the order device d runs its tasks under the
    interleaved schedule: micro-batches in groups of pp; within a group the forwards take the
    device's chunks in ascending order (each chunk: the pp micro-batches of the group), the
    backwards in descending order; 2 (pp - d - 1) + (chunks - 1) pp warm-up forwards, then one
    forward / one backward, then the remaining backwards."""
    fwd, bwd = [], []
    for g in range(m // pp):
        for ch in range(chunks):
            for r in range(pp):
                fwd.append((0, ch * pp + d, g * pp + r))
        for ch in reversed(range(chunks)):
            for r in range(pp):
                bwd.append((1, ch * pp + d, g * pp + r))
    n = len(fwd)
    w = min(2 * (pp - d - 1) + (chunks - 1) * pp, n)
    order = fwd[:w]
    f, b = w, 0
    while f < n:
        order.append(fwd[f]); f += 1
        order.append(bwd[b]); b += 1
    order += bwd[b:]
    return order


def idle_before_lists(start: np.ndarray, end: np.ndarray, lists) -> np.ndarray:
    """The same for an explicit schedule: lists[d] = [(kind, virtual stage, micro-batch)] is the order
    in which device d runs its tasks.  Entries of tasks that no list holds stay zero."""
    out = np.zeros_like(start)
    for lst in lists:
        prev_end = 0
        for kind, k, j in lst:
            out[kind, k, j] = int(start[kind, k, j]) - prev_end
            prev_end = int(end[kind, k, j])
    return out


def idle_before(start: np.ndarray, end: np.ndarray, schedule: int, chunks: int = 1) -> np.ndarray:
    """start, end [2][stages][m] of one candidate -> idle time in front of every stage-task, same
    shape; stages = pp, or pp * chunks virtual stages for the interleaved schedule (3)."""
    _, S, m = start.shape
    out = np.zeros_like(start)
    if schedule == 3:
        pp = S // chunks
        for d in range(pp):
            prev_end = 0
            for kind, k, j in device_order_interleaved(pp, m, chunks, d):
                out[kind, k, j] = int(start[kind, k, j]) - prev_end
                prev_end = int(end[kind, k, j])
        return out
    pp = S
    for s in range(pp):
        prev_end = 0
        for kind, j in device_order(pp, m, schedule, s):
            out[kind, s, j] = int(start[kind, s, j]) - prev_end
            prev_end = int(end[kind, s, j])
    return out
