"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (signed overflow, shifts, misaligned
and out-of-bounds accesses trap).  CPU only; no GPU code runs.

 * the oracle: oracle/distsim_oracle.c is built with gcc -fsanitize=address,undefined together with
   tests/sanitize/oracle_driver.c, which feeds it workload files written here (all the kinds of
   candidates the interface takes, valid and not) from exact-size heap buffers; its outputs must
   hash to what the ordinary build of the oracle returns, and no sanitizer report may appear;
 * the library: the host side of csrc/distsim.hip (size queries, carving of the workspace and of
   distsim_events, argument checks) is built with the sanitizers on the host compiler only and driven
   by tests/sanitize/library_host_driver.cpp.
"""
import os
import subprocess

import numpy as np
import pytest

from helpers import mk, mk_cluster, mk_costs
from workloads import make_workload, subset

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _fnv(a) -> str:
    h = 1469598103934665603
    for b in np.ascontiguousarray(a).tobytes():
        h = ((h ^ b) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return f"{h:016x}"


def _write(path, w, timeline=False):
    co, cl, ca = w.costs, w.cluster, w.cand
    C = len(ca["pp"])
    pool = np.ascontiguousarray(ca["part_pool"], np.uint8)
    soff = ca.get("schedule_off")
    words = ca.get("schedule_words")
    ns = len(soff) - 1 if soff is not None else 0
    hdr = np.asarray([co["L"], co["V"], cl["num_devices"], cl["gpus_per_node"], *cl["alpha_ns"], *cl["beta_bytes_per_ns"],
                      cl["dp_bucket_bytes"], cl.get("p2p_blocking", 0), C, pool.size, ns,
                      0 if words is None else len(words), int(ca.get("chunks") is not None), int(timeline)], np.int64)
    with open(path, "wb") as f:
        f.write(hdr.tobytes())
        f.write(np.ascontiguousarray(co["variant_tp"], np.int32).tobytes())
        for k in ("fwd_comp_ns", "bwd_comp_ns", "fwd_comm_ns", "bwd_comm_ns", "act_bytes", "grad_bytes", "a2a_bytes"):
            f.write(np.ascontiguousarray(co[k], np.int64).tobytes())
        for k in ("dp", "tp", "pp", "m"):
            f.write(np.ascontiguousarray(ca[k], np.int32).tobytes())
        f.write(np.ascontiguousarray(ca["schedule"], np.uint8).tobytes())
        f.write(np.ascontiguousarray(ca["chunks"] if ca.get("chunks") is not None else np.zeros(C), np.int32).tobytes())
        f.write(np.ascontiguousarray(ca["part_off"], np.int64).tobytes())
        f.write(pool.tobytes())
        f.write(np.ascontiguousarray(soff if soff is not None else [0], np.int64).tobytes())
        if words is not None:
            f.write(np.ascontiguousarray(words, np.int32).tobytes())


def _workloads():
    """Small lists of every kind: the seeded configurations, ragged shapes, every schedule, the three p2p
    readings, buckets, invalid candidates, partitions that run off the pool, explicit schedules."""
    from test_explicit_schedule_pins import random_schedule
    from workloads.schedules import chain, dapple_lists, interleaved_lists, interleaved_stages, pack_schedule, pack_schedules
    rng = np.random.default_rng(2306)
    out = [make_workload("tiny"), make_workload("gpt24")]
    w = make_workload("gpt96")
    out.append(subset(w, rng.choice(w.C, 300, replace=False)))
    w = make_workload("hetero64", C=2000)
    out.append(subset(w, np.arange(0, 2000, 7)))
    L = 40
    for blocking, bucket in ((0, 0), (1, 1 << 14), (2, 0)):
        costs = mk_costs(rng.integers(0, 5000, (2, L)).tolist(), rng.integers(0, 9000, (2, L)).tolist(),
                         fa=rng.integers(0, 300, (2, L)).tolist(), ba=rng.integers(0, 300, (2, L)).tolist(),
                         act=(rng.integers(0, 100, (2, L)) * 64).tolist(), grad=rng.integers(0, 1 << 16, (2, L)).tolist(),
                         a2a=(rng.integers(0, 3, (2, L)) * 4096).tolist(), tps=(1, 2))
        N = 2 * 3 * 4 * 5 * 7
        rows, blocks = [], []
        for _ in range(150):
            pp = int(rng.choice([d for d in range(1, 41) if N % d == 0] + [50, 70]))
            tp = int(rng.choice([1, 2, 5]))
            dp = max(N // (pp * tp), 1)
            m = int(rng.choice([1, 2, 3, 8, 33]))
            sc = int(rng.choice([0, 1, 2, 3, 4, 7]))
            v = int(rng.integers(1, 4))
            S = pp * v if sc == 3 else pp
            bnd = None
            if rng.random() < 0.5 and 1 <= S <= L:
                bnd = [0] + np.sort(rng.choice(np.arange(1, L), S - 1, replace=False)).tolist() + [L]
                if rng.random() < 0.1:
                    bnd = bnd[:-2] + [L]                       # one boundary short: the partition runs off the pool
            if sc == 3 and rng.random() < 0.7:
                m = pp * int(rng.integers(1, 3))
            ident = v
            if sc == 4:
                if rng.random() < 0.5 and pp <= 8:
                    place, prev, lists = random_schedule(rng, pp, int(rng.integers(1, 9)), m)
                    blocks.append(pack_schedule(pp, list(zip(place, [0] * len(place), prev)), m, 1, int(rng.integers(1, 3)), lists))
                elif m % pp == 0 and pp * 2 <= L:
                    blocks.append(pack_schedule(pp, interleaved_stages(pp, 2), m, 2 * pp, 1, interleaved_lists(pp, 2, m)))
                else:
                    blocks.append(pack_schedule(pp, chain(pp), m, pp, 1, dapple_lists(pp, m))[: None if rng.random() < 0.8 else -2])
                ident = len(blocks) - 1 if rng.random() < 0.9 else len(blocks) + 3
            rows.append((dp, tp, pp, m, sc, bnd, ident))
        w = mk(costs, mk_cluster(N, g=int(rng.choice([1, 4, 8])), bucket=bucket, blocking=blocking), rows)
        w.cand["part_off"][::17] = rng.integers(-3, len(w.cand["part_pool"]) + 5, len(w.cand["part_off"][::17]))
        w.cand["schedule_off"], w.cand["schedule_words"] = pack_schedules(blocks)
        out.append(w)
    return out


def test_oracle_under_address_and_undefined_behaviour_sanitizers(oracle_mod, tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["gcc", *SAN, "-fopenmp", "-Wall", "-o", str(exe), os.path.join(ROOT, "oracle", "distsim_oracle.c"),
                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")])
    n_ok = 0
    for i, w in enumerate(_workloads()):
        runs = [(w, False)]
        ok = np.nonzero(oracle_mod.simulate(w)["status"] == 0)[0]
        runs += [(subset(w, [int(c)]), True) for c in ok[:: max(1, len(ok) // 5)][:5]]      # single candidates with the timeline
        for j, (x, tl) in enumerate(runs):
            path = tmp_path / f"w{i}_{j}.bin"
            _write(path, x, tl)
            res = subprocess.run([str(exe), str(path)], capture_output=True, text=True, env=ENV)
            assert res.returncode == 0 and "runtime error" not in res.stderr and "Sanitizer" not in res.stderr, res.stderr[-3000:]
            got = dict(line.split() for line in res.stdout.splitlines())
            want = oracle_mod.simulate(x, nthreads=1, timeline=tl)
            keys = ["status", "batch_ns", "num_events", "stage_off", "comp_busy_ns", "comm_busy_ns", "util"]
            keys += ["start", "end", "ar_window"] if tl else []
            for k in keys:
                assert got[k] == _fnv(want[k]), (i, j, k)
            st = oracle_mod.stage_table(x, want)
            for k in ("tab", "layer_lo", "layer_hi"):
                assert got[k] == _fnv(st[k]), (i, j, k)
            wgt = x.cand["dp"].astype(np.int64) * x.cand["m"]
            assert got["best0"] == _fnv(np.asarray(oracle_mod.search(want["batch_ns"]), np.int64))
            assert got["best1"] == _fnv(np.asarray(oracle_mod.search(want["batch_ns"], wgt, 1), np.int64))
            n_ok += int((want["status"] == 0).sum())
    assert n_ok > 1000


def test_library_host_code_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not (os.path.exists(hipcc) and os.path.exists(clangxx)):
        pytest.skip("no ROCm toolchain here")
    obj = tmp_path / "distsim_san.o"
    host = [x for f in SAN if f.startswith("-fsan") or f.startswith("-fno-san") for x in ("-Xarch_host", f)]
    r = subprocess.run([hipcc, "-O1", "-g", "-std=c++17", *host, "-I" + os.path.join(ROOT, "include"),
                        "-I" + os.path.join(ROOT, "paper_2306_08423_amd", "csrc"),
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                        "--offload-arch=gfx950", "-c", os.path.join(ROOT, "paper_2306_08423_amd", "csrc", "distsim.hip"),
                        "-o", str(obj)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = tmp_path / "library_host_san"
    subprocess.check_call([clangxx, *SAN, "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize", "library_host_driver.cpp"), str(obj),
                           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)])
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0")        # the HIP runtime's own start-up allocations are not ours to judge
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert res.returncode == 0 and "library host checks passed" in res.stdout, res.stdout[-2000:] + res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "Sanitizer" not in res.stderr, res.stderr[-3000:]
