"""Are the pins sharp?  Each case plants one plausible mistake in a COPY of the oracle's source (on
the CPU, in a temporary directory), builds it, points the oracle's front end at the mutant and runs
the pins: at least one of them has to fail.  The real oracle is restored afterwards."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_device_buckets_pins as bpins
import test_explicit_schedule_pins as xpins
import test_oracle_pins as pins
import test_stage_table_pins as spins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "distsim_oracle.c")

MUTANTS = [
    ("warm-up one deeper", "int w = pp - 1 - s;", "int w = pp - s;"),
    ("warm-up one shallower", "int w = pp - 1 - s;", "int w = pp - 2 - s; if (w < 0) w = 0;"),
    ("p2p bytes of the wrong layer", "int64_t bytes = act[bnd[s + 1] - 1];", "int64_t bytes = act[bnd[s + 1] < L ? bnd[s + 1] : L - 1];"),
    ("forward p2p latency dropped", "int64_t arrive = now + pf[s];", "int64_t arrive = now;"),
    ("backward p2p latency dropped", "int64_t arrive = now + pb[s];", "int64_t arrive = now;"),
    ("ring volume without the factor 2", "(2ull * (uint64_t)(n - 1) * (uint64_t)bytes)", "((uint64_t)(n - 1) * (uint64_t)bytes)"),
    ("ring volume with N instead of N-1", "(2ull * (uint64_t)(n - 1) * (uint64_t)bytes)", "(2ull * (uint64_t)n * (uint64_t)bytes)"),
    ("collective link class off by one", "int k = n <= cl->gpus_per_node ? 0 : 1;\n    return cl->alpha[k] + (int64_t)((2ull",
     "int k = n < cl->gpus_per_node ? 0 : 1;\n    return cl->alpha[k] + (int64_t)((2ull"),
    ("p2p link class ignores dp", "int64_t na = ((int64_t)s * tp * dp) / g, nb = ((int64_t)(s + 1) * tp * dp) / g;",
     "int64_t na = ((int64_t)s * tp) / g, nb = ((int64_t)(s + 1) * tp) / g;"),
    ("tp all-reduce also for tp = 1", "if (tp > 1) { t += fa[l]; mb_[s__] += fa[l]; }", "{ t += fa[l]; mb_[s__] += fa[l]; }"),
    ("backward all-reduce forgotten", "if (tp > 1) { t += ba[l]; mb_[s__] += ba[l]; }", "if (tp > 1) { mb_[s__] += ba[l]; }"),
    ("p2p not counted as communication", "mb_[s] += pf[s]; nev++;", "nev++;"),
    ("all-reduce starts at time zero", "heap_push(h, now + d, EV_AR_DONE, s, 0, 0);", "heap_push(h, d, EV_AR_DONE, s, 0, 0);"),
    ("last bucket dropped", "if (e.layer == bnd[s] && acc[s] > 0) {", "if (0 && e.layer == bnd[s] && acc[s] > 0) {"),
    ("buckets do not queue", "int64_t st = comm_free[s] > now ? comm_free[s] : now;\n                comm_free[s] = st + d;\n                heap_push(h, comm_free[s], EV_AR_DONE, s, 0, 0);\n                mb_[s] += d;\n                if (tl_ar) { if (tl_ar[s] < 0) tl_ar[s] = st; tl_ar[pp + s] = comm_free[s]; }\n                acc[s] -= cap;",
     "int64_t st = now;\n                comm_free[s] = st + d;\n                heap_push(h, comm_free[s], EV_AR_DONE, s, 0, 0);\n                mb_[s] += d;\n                if (tl_ar) { if (tl_ar[s] < 0) tl_ar[s] = st; tl_ar[pp + s] = comm_free[s]; }\n                acc[s] -= cap;"),
    ("gradients of every micro-batch", "int last_bwd = (kd == 1 && next[s__] == 2 * m - 1);", "int last_bwd = (kd == 1);"),
    ("async schedule keeps the all-reduce", "const int sync = sched != 2;", "const int sync = 1;"),
    ("blocking send not on the device", "if (cl->p2p_blocking == 1) {      /* the send runs on the device */", "if (0) {"),
    ("links do not serialise", "int64_t depart = now > link_f[s] ? now : link_f[s];", "int64_t depart = now;"),
    ("all-to-all volume without (n-1)/n", "(((uint64_t)(n - 1) * (uint64_t)bytes) / ((uint64_t)n * (uint64_t)cl->beta[k]))", "((uint64_t)bytes / (uint64_t)cl->beta[k])"),
    ("GPipe backward before the last forward", "for (int i = 0; i < m; i++) { k[n] = 0; j[n++] = i; }\n            for (int i = 0; i < m; i++) { k[n] = 1; j[n++] = i; }",
     "for (int i = 0; i < m - 1; i++) { k[n] = 0; j[n++] = i; }\n            k[n] = 1; j[n++] = 0; k[n] = 0; j[n++] = m - 1;\n            for (int i = 1; i < m; i++) { k[n] = 1; j[n++] = i; }"),
    ("interleaved: warm-up of the plain schedule", "int64_t W = 2ll * (pp - d - 1) + (int64_t)(vch - 1) * pp;", "int64_t W = (pp - d - 1) + (int64_t)(vch - 1) * pp;"),
    ("interleaved: backward chunks not mirrored", "kk[n] = 1; vs[n] = (int32_t)((vch - 1 - w__ / pp) * pp + d);", "kk[n] = 1; vs[n] = (int32_t)((w__ / pp) * pp + d);"),
    ("interleaved: micro-batch groups ignored", "jj[n] = (int32_t)((i__ / ((int64_t)pp * vch)) * pp + w__ % pp); n++; } while (0)\n#define PUT_B", "jj[n] = (int32_t)(w__ % pp); n++; } while (0)\n#define PUT_B"),
    ("interleaved: link class by virtual stage", "int64_t na = ((int64_t)(k % pp) * tp * dp) / g, nb = ((int64_t)((k + 1) % pp) * tp * dp) / g;", "int64_t na = ((int64_t)k * tp * dp) / g, nb = ((int64_t)(k + 1) * tp * dp) / g;"),
    ("interleaved: all-reduce of one chunk only", "for (int c = 0; c < vch; c++)\n                    for (int l = bnd[c * pp + d]; l < bnd[c * pp + d + 1]; l++) G += grad[l];", "for (int c = 0; c < 1; c++)\n                    for (int l = bnd[c * pp + d]; l < bnd[c * pp + d + 1]; l++) G += grad[l];"),
    ("explicit: backward of a last stage does not wait for its forward", "(next[k] < 0 ? doneF[(int64_t)k * m + j] : sc->arrB[(int64_t)k * m + j])", "(next[k] < 0 ? 1 : sc->arrB[(int64_t)k * m + j])"),
    ("explicit: p2p of the receiving part", "int64_t t = p2p_ns(cl, act[bnd[part[q] + 1] - 1], na == nb ? 0 : 1);", "int64_t t = p2p_ns(cl, act[bnd[part[k] + 1] - 1], na == nb ? 0 : 1);"),
    ("explicit: link class by stage number", "int64_t na = ((int64_t)place[q] * tp * dp) / g, nb = ((int64_t)place[k] * tp * dp) / g;", "int64_t na = ((int64_t)q * tp * dp) / g, nb = ((int64_t)k * tp * dp) / g;"),
    ("explicit: all-reduce ignores the replicas", "int64_t dd = allreduce_ns(cl, (int64_t)dp * replicas, G);", "int64_t dd = allreduce_ns(cl, (int64_t)dp, G);"),
    ("explicit: gradient bytes of every stage on every device", "for (int q = 0; q < S; q++) if (place[q] == d)\n                    for (int l = bnd[part[q]]", "for (int q = 0; q < S; q++)\n                    for (int l = bnd[part[q]]"),
    ("explicit: latency of the backward edge dropped", "int64_t arrive = now + pb[k];\n                if (cl->p2p_blocking == 1) arrive = now;\n                if (cl->p2p_blocking == 2) {\n                    int64_t *lf = &link_free[(int64_t)d * pp + place[prev[k]]];",
     "int64_t arrive = now;\n                if (cl->p2p_blocking == 1) arrive = now;\n                if (cl->p2p_blocking == 2) {\n                    int64_t *lf = &link_free[(int64_t)d * pp + place[prev[k]]];"),
    ("explicit: links do not serialise", "int64_t *lf = &link_free[(int64_t)d * pp + place[next[k]]];\n                        int64_t depart = now > *lf ? now : *lf;",
     "int64_t *lf = &link_free[(int64_t)d * pp + place[next[k]]];\n                        int64_t depart = now;"),
    ("explicit: one queue per sending device, whatever the receiver", "int64_t *lf = &link_free[(int64_t)d * pp + place[prev[k]]];", "int64_t *lf = &link_free[(int64_t)d * pp];"),
    ("explicit: one queue per receiving device, whatever the sender", "int64_t *lf = &link_free[(int64_t)d * pp + place[next[k]]];", "int64_t *lf = &link_free[place[next[k]]];"),
    ("interleaved: links do not serialise", "int64_t *lf = &link_free[(int64_t)d * pp + (k + 1) % pp];\n                    int64_t depart = now > *lf ? now : *lf;",
     "int64_t *lf = &link_free[(int64_t)d * pp + (k + 1) % pp];\n                    int64_t depart = now;"),
    ("interleaved: a queue per chunk boundary instead of per pair of devices", "int64_t *lf = &link_free[(int64_t)d * pp + (k - 1) % pp];", "int64_t *lf = &link_free[(int64_t)(k % (pp * pp))];"),
    ("stage table: p2p bytes of the next stage's first layer", "PF = p2p_ns(&cl, act[(int64_t)v * L + hi - 1],", "PF = p2p_ns(&cl, act[(int64_t)v * L + (hi < L ? hi : L - 1)],"),
    ("stage table: backward p2p with the class of the other boundary", "((s - 1) * per) / g == (s * per) / g ? 0 : 1", "(s * per) / g == ((s + 1) * per) / g ? 0 : 1"),
    ("stage table: all-reduce column for the asynchronous schedule", "tab[7 * n + i] = schedule[c] == 2 ? 0 : allreduce_ns(&cl, dp[c], G);", "tab[7 * n + i] = allreduce_ns(&cl, dp[c], G);"),
    ("stage table: all-reduce events of a tp = 1 layer", "if (tp[c] > 1) { FA += fa[x]; BA += ba[x]; }", "{ FA += fa[x]; BA += ba[x]; }"),
    ("stage table: all-to-all in the forward pass only", "                BA += alltoall_ns(&cl, dp[c], a2a[x]);\n", ""),
    ("stage table: stage bounds of the uniform split rounded up", "(int)(((int64_t)(s + 1) * L) / P);\n            const int64_t i", "(int)(((int64_t)(s + 1) * L + P - 1) / P);\n            const int64_t i"),
    ("device buckets: gradients of every micro-batch", "if (j == m - 1 && cap > 0 && dp > 1)", "if (cap > 0 && dp > 1)"),
    ("device buckets: gradients of the first micro-batch", "if (j == m - 1 && cap > 0 && dp > 1)", "if (j == 0 && cap > 0 && dp > 1)"),
    ("device buckets: what is left after the last gradient is dropped", "while (acc[d] >= cap || (pend[d] == 0 && acc[d] > 0)) {", "while (acc[d] >= cap) {"),
    ("device buckets: what is left goes after every chunk", "            pend[d]--;\n            while (acc[d] >= cap || (pend[d] == 0 && acc[d] > 0)) {",
     "            pend[d] = e.layer == bnd[k] ? 0 : 1;\n            while (acc[d] >= cap || (pend[d] == 0 && acc[d] > 0)) {"),
    ("device buckets: events do not queue", "int64_t st = comm_free[d] > now ? comm_free[d] : now;", "int64_t st = now;"),
    ("device buckets: the trailing event stays", "if (next[d] == per_dev && dp > 1 && cap == 0) {", "if (next[d] == per_dev && dp > 1) {"),
    ("device buckets, explicit: the first backward of a stage instead of the last", "if (x >> 31) last_bwd[(x >> 16) & 0x7fff] = i;",
     "if ((x >> 31) && last_bwd[(x >> 16) & 0x7fff] < 0) last_bwd[(x >> 16) & 0x7fff] = i;"),
    ("device buckets, explicit: the replicas are forgotten", "int64_t dd = allreduce_ns(cl, ranks, bytes);", "int64_t dd = allreduce_ns(cl, dp, bytes);"),
    ("device buckets, explicit: stages without backward keep the device waiting", "if (last_bwd[q] >= 0) pend[place[q]] +=", "pend[place[q]] +="),
    ("utilisation from communication", "util[s] = now > 0 ? (double)cb[s] / (double)now : 0.0;", "util[s] = now > 0 ? (double)mb_[s] / (double)now : 0.0;"),
]

# pins that take only the oracle module (parametrised ones are called with one or two settings)
PINS = [
    lambda o: pins.test_golden_pp2_m4_timeline(o, 1_000_000, 2_025_000, 5000, 4 << 20),
    lambda o: pins.test_golden_pp2_m4_timeline(o, 5, 11, 1, 200 * 13),
    pins.test_golden_tiny_numbers,
    pins.test_golden_bucketed_allreduce,
    lambda o: pins.test_uniform_pipeline_closed_form(o, 0),
    lambda o: pins.test_uniform_pipeline_closed_form(o, 1),
    pins.test_gpipe_flow_shop_closed_form,
    pins.test_brute_force_longest_path_all_timestamps,
    pins.test_blocking_p2p_against_task_graph,
    pins.test_serialised_links_against_graph_with_send_nodes,
    lambda o: pins.test_inflight_bound_of_early_backward(o, 4, 8),
    pins.test_ring_allreduce_volume,
    pins.test_p2p_link_class_and_alltoall,
    pins.test_model_parallel_mapping,
    pins.test_metamorphic,
    pins.test_dp_changes_only_the_tail,
    pins.test_async_schedule_is_dapple_without_the_global_sync,
    lambda o: pins.test_invariants_on_workloads(o, "gpt24"),
    pins.test_interleaved_uniform_closed_form,
    pins.test_interleaved_against_task_graph,
    pins.test_interleaved_validity_rules,
    pins.test_interleaved_link_classes_follow_the_devices,
    xpins.test_builtin_schedules_written_out_as_lists,
    xpins.test_random_schedules_against_the_task_graph,
    xpins.test_serialised_links_against_graph_with_send_nodes,
    xpins.test_bidirectional_lists_run_and_use_both_directions,
    xpins.test_invalid_explicit_schedules,
    bpins.test_two_chunks_on_one_device_by_hand,
    bpins.test_lists_of_the_built_in_schedules_with_buckets,
    bpins.test_bucket_chain_of_interleaved_candidates_from_the_dump,
    bpins.test_a_stage_without_backward_gives_no_gradient_with_buckets,
    bpins.test_replicas_enter_the_bucket_events,
    spins.test_tiny_golden_stage_events,
    spins.test_every_column_against_discrete_event_timelines,
    lambda o: spins.test_busy_time_identities(o, "gpt24"),
]


def _caught(mod) -> bool:
    for pin in PINS:
        try:
            pin(mod)
        except AssertionError:
            return True
        except Exception:          # a mutant may also crash a pin's bookkeeping (index, key): caught as well
            return True
    return False


def test_every_pin_passes_on_the_real_oracle(oracle_mod):
    assert not _caught(oracle_mod)


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(oracle_mod, tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site not found: {name}"
    mutated = text.replace(old, new, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / "libmutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-w", "-o", str(so), str(c)])
    real = oracle._load()
    mutant = ctypes.CDLL(str(so))
    mutant.oracle_simulate.restype = ctypes.c_int
    mutant.oracle_search.restype = ctypes.c_int
    mutant.oracle_stage_table.restype = ctypes.c_int
    oracle._lib = mutant
    try:
        assert _caught(oracle_mod), f"no pin notices: {name}"
    finally:
        oracle._lib = real
