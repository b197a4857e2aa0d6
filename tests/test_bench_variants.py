"""The variant workloads that bench.py times are real work: the oracle accepts every candidate
that a variant hands to its kernel."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import bench  # noqa: E402
import oracle  # noqa: E402
from workloads import make_workload  # noqa: E402


def test_variant_workloads_are_valid():
    w = make_workload("gpt48")
    names = []
    for name, wv, kernel, counted in bench.variant_workloads(w, 600):
        r = oracle.simulate(wv, nthreads=4)
        ok = r["status"] == 0
        assert counted.sum() > 50, name
        assert (ok | ~counted).all(), name
        sched = wv.cand["schedule"]
        want = {"asynchronous": 2, "interleaved_2_chunks": 3, "explicit_lists": 4}.get(name)
        if want is not None:
            assert (sched[counted] == want).all() and not (sched[~counted] == want).any()
        names.append((name, kernel))
    assert names == [("default", "k_simulate"), ("p2p_blocking_1", "k_simulate"), ("serialised_links", "k_simulate"),
                     ("asynchronous", "k_simulate"), ("interleaved_2_chunks", "k_simulate_virtual"),
                     ("explicit_lists", "k_simulate_explicit")]
