"""Explicit pipeline schedules: the input S of Algorithm 1 written out (Sec. 4.3: which device runs
which stage-task of which micro-batch, in which order).  Inputs only, no timing arithmetic: task
lists from the schedules' definitions and the packing into the 32-bit words that the library and
the oracle read.

A schedule is (pp, stages, m, nparts, replicas, lists):
  stages  list over virtual stages k of (device, part, prev): the device that holds the stage, the
          part of the layer partition it computes, the stage before it in its pipeline (-1: first)
  lists   list over devices of [(kind, stage, micro-batch)] in execution order, kind 0 = forward
"""
from __future__ import annotations

import numpy as np

FWD, BWD = 0, 1


def pack_schedule(pp: int, stages, m: int, nparts: int, replicas: int, lists) -> np.ndarray:
    """The block of 32-bit words of one schedule:
    pp, S, m, nparts, replicas | first task of every device's list, task total | per stage
    (device, part, prev) | tasks kind << 31 | stage << 16 | micro-batch."""
    assert len(lists) == pp
    S = len(stages)
    off = [0]
    for lst in lists:
        off.append(off[-1] + len(lst))
    words = [pp, S, m, nparts, replicas] + off
    for dev, part, prev in stages:
        words += [dev, part, prev]
    out = np.asarray(words, dtype=np.int64)
    tasks = np.asarray([(kd << 31) | (k << 16) | j for lst in lists for kd, k, j in lst], dtype=np.int64)
    w = np.concatenate([out, tasks]).astype(np.uint32).view(np.int32) if len(tasks) else out.astype(np.int32)
    return np.ascontiguousarray(w)


def unpack_schedule(words):
    """Inverse of pack_schedule: (pp, stages, m, nparts, replicas, lists)."""
    w = np.asarray(words).astype(np.int64)
    pp, S, m, nparts, replicas = (int(x) for x in w[:5])
    off = w[5:5 + pp + 1]
    st = w[5 + pp + 1:5 + pp + 1 + 3 * S].reshape(S, 3)
    tasks = w[5 + pp + 1 + 3 * S:] & 0xffffffff
    lists = [[(int(x >> 31), int((x >> 16) & 0x7fff), int(x & 0xffff)) for x in tasks[off[d]:off[d + 1]]] for d in range(pp)]
    return pp, [tuple(int(v) for v in r) for r in st], m, nparts, replicas, lists


def pack_schedules(blocks):
    """Offsets [n + 1] and the word pool of several schedules."""
    off = np.zeros(len(blocks) + 1, np.int64)
    for i, b in enumerate(blocks):
        off[i + 1] = off[i] + len(b)
    words = np.concatenate(blocks).astype(np.int32) if blocks else np.zeros(0, np.int32)
    return off, words


def chain(pp: int):
    """One pipeline over pp devices, stage s on device s with part s."""
    return [(s, s, s - 1) for s in range(pp)]


def gpipe_lists(pp: int, m: int):
    """All forwards, then all backwards, in micro-batch order (Sec. 2.1.3)."""
    return [[(FWD, s, j) for j in range(m)] + [(BWD, s, j) for j in range(m)] for s in range(pp)]


def dapple_lists(pp: int, m: int):
    """Early backward: stage s keeps at most pp - s micro-batches in flight, i.e. min(pp - 1 - s, m)
    warm-up forwards, then one forward / one backward, then the remaining backwards."""
    lists = []
    for s in range(pp):
        w = min(pp - 1 - s, m)
        lst = [(FWD, s, j) for j in range(w)]
        f, b = w, 0
        while f < m:
            lst.append((FWD, s, f)); f += 1
            lst.append((BWD, s, b)); b += 1
        lst += [(BWD, s, j) for j in range(b, m)]
        lists.append(lst)
    return lists


def interleaved_stages(pp: int, chunks: int):
    """Virtual stage k = chunk * pp + device computes part k; one pipeline through all of them."""
    return [(k % pp, k, k - 1) for k in range(pp * chunks)]


def interleaved_lists(pp: int, chunks: int, m: int):
    """Interleaved one-forward-one-backward (m a multiple of pp): per device, micro-batches in groups
    of pp; within a group the forwards take the device's chunks in ascending order, the backwards
    in descending order; 2 (pp - d - 1) + (chunks - 1) pp warm-up forwards."""
    assert m % pp == 0
    lists = []
    for d in range(pp):
        fwd, bwd = [], []
        for g in range(m // pp):
            for ch in range(chunks):
                fwd += [(FWD, ch * pp + d, g * pp + r) for r in range(pp)]
            for ch in reversed(range(chunks)):
                bwd += [(BWD, ch * pp + d, g * pp + r) for r in range(pp)]
        n = len(fwd)
        w = min(2 * (pp - d - 1) + (chunks - 1) * pp, n)
        lst = fwd[:w]
        f, b = w, 0
        while f < n:
            lst.append(fwd[f]); f += 1
            lst.append(bwd[b]); b += 1
        lst += bwd[b:]
        lists.append(lst)
    return lists


def bidirectional_stages(pp: int):
    """Two pipelines over the same pp devices in opposite directions, each a full replica of the
    model: stage s of the first on device s, stage s of the second (virtual stage pp + s) on
    device pp - 1 - s; both compute part s."""
    down = [(s, s, s - 1) for s in range(pp)]
    up = [(pp - 1 - s, s, pp + s - 1 if s > 0 else -1) for s in range(pp)]
    return down + up


def bidirectional_lists(pp: int, m: int):
    """A schedule in the manner of bidirectional pipelines (two replicas, gradient all-reduce over
    dp * 2 ranks): micro-batches with an even index go down, the others up; each pipeline keeps the
    early-backward order of its own micro-batches, and a device merges its two lists by the slot
    numbers that order gives with unit task lengths (ties: the first pipeline first).  An input
    generator for tests and benchmarks, not a statement about any published schedule."""
    halves = [[j for j in range(m) if j % 2 == 0], [j for j in range(m) if j % 2 == 1]]
    per_dev = [[] for _ in range(pp)]
    for pipe, mbs in enumerate(halves):
        n = len(mbs)
        for s in range(pp):
            dev = s if pipe == 0 else pp - 1 - s
            k = s + pipe * pp
            w = min(pp - 1 - s, n)
            for i, j in enumerate(mbs):
                slot_f = s + i if i <= w else s + 2 * i
                slot_b = 2 * pp - 1 - s + 2 * i
                per_dev[dev].append((slot_f, pipe, FWD, k, j))
                per_dev[dev].append((slot_b, pipe, BWD, k, j))
    return [[(kd, k, j) for _, _, kd, k, j in sorted(lst)] for lst in per_dev]
