"""Seeded generators for the five synthetic evaluation workloads.

Every workload is a triple (cost table, cluster, candidate list):

* cost table   -- per (tensor-parallel variant, layer) event times in integer
                  nanoseconds and message sizes in bytes; stands in for the
                  output of DistSim's event profiler (Sec. 4.2), which needs
                  real GPUs.  Compute times come from the FLOPs/peak heuristic
                  of Sec. 2.3 perturbed by a log-normal efficiency; the
                  in-layer tensor-parallel all-reduce time is drawn from an
                  alpha-beta ring model with the per-device volume of Sec. 4.2.
* cluster      -- simulated device count, node size, link alpha/beta.
* candidates   -- struct-of-arrays list of hybrid strategies "xM xP xD"
                  (Sec. 5.1 notation) x micro-batch count x schedule x
                  layer-to-stage partition, as in the grid search of Sec. 6.

Random numbers come from numpy's Philox counter-based generator
(``numpy.random.Philox``) keyed with ``2306084230 + k`` for workload k.  Tables
are drawn once on the host and handed unchanged to whoever consumes them, so the
floating-point used here can never cause a mismatch between two consumers.

Nothing in this file evaluates a schedule, a timeline or a candidate.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 2306084230
CONFIG_NAMES = ("tiny", "tiny_b", "gpt24", "gpt48", "gpt96", "hetero64")

PEAK_FLOPS = 150.0e12          # A40-class dense fp16 peak, a free parameter
INTRA = (5_000, 200)           # alpha ns, beta bytes/ns (200 GB/s)
INTER = (10_000, 25)           # alpha ns, beta bytes/ns (25 GB/s)
GPUS_PER_NODE = 8
MIB = 1 << 20


@dataclass
class Workload:
    name: str
    costs: Dict[str, np.ndarray]        # see _empty_costs for the keys
    cluster: Dict[str, object]
    cand: Dict[str, np.ndarray]         # dp,tp,pp,m int32; schedule u8; part_off i64; part_pool u8
    notes: str = ""
    meta: Dict[str, object] = field(default_factory=dict)

    @property
    def C(self) -> int:
        return int(self.cand["dp"].shape[0])

    @property
    def L(self) -> int:
        return int(self.costs["L"])

    @property
    def V(self) -> int:
        return int(self.costs["V"])


def _rng(k: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=BASE_SEED + k))


def _cluster(num_devices: int, bucket: int = 0) -> Dict[str, object]:
    return {
        "num_devices": int(num_devices),
        "gpus_per_node": GPUS_PER_NODE,
        "alpha_ns": (INTRA[0], INTER[0]),
        "beta_bytes_per_ns": (INTRA[1], INTER[1]),
        "dp_bucket_bytes": int(bucket),
    }


def _empty_costs(L: int, tps: Tuple[int, ...]) -> Dict[str, np.ndarray]:
    V = len(tps)
    z = lambda: np.zeros((V, L), dtype=np.int64)
    return {
        "L": L, "V": V,
        "variant_tp": np.asarray(tps, dtype=np.int32),
        "fwd_comp_ns": z(), "bwd_comp_ns": z(),
        "fwd_comm_ns": z(), "bwd_comm_ns": z(),
        "act_bytes": z(), "grad_bytes": z(), "a2a_bytes": z(),
    }


def _profiled_tp_allreduce_ns(n: int, nbytes: int) -> int:
    """Stand-in for a *profiled* tensor-parallel all-reduce event (input recipe)."""
    if n == 1:
        return 0
    a, b = INTRA if n <= GPUS_PER_NODE else INTER
    return a + (2 * (n - 1) * nbytes) // (n * b)


def _transformer_costs(rng, L: int, h: int, s: int, tps: Tuple[int, ...],
                       scale: np.ndarray | None = None) -> Dict[str, np.ndarray]:
    """fwd = layer FLOPs / (tp * peak * eff), eff ~ lognormal(ln 0.5, 0.1) per (variant, layer)."""
    c = _empty_costs(L, tps)
    V = len(tps)
    flops = 24.0 * s * h * h + 4.0 * s * s * h
    eff = rng.lognormal(mean=np.log(0.5), sigma=0.1, size=(V, L))
    jitter = rng.integers(0, 50_001, size=(V, L), dtype=np.int64)
    mult = np.ones(L) if scale is None else np.asarray(scale, dtype=np.float64)
    for v, tp in enumerate(tps):
        sec = flops * mult / (tp * PEAK_FLOPS * eff[v])
        fc = np.floor(sec * 1e9).astype(np.int64)
        c["fwd_comp_ns"][v] = fc
        c["bwd_comp_ns"][v] = 2 * fc + jitter[v]
        ar = 2 * _profiled_tp_allreduce_ns(tp, s * h * 2)
        c["fwd_comm_ns"][v] = ar
        c["bwd_comm_ns"][v] = ar
        c["act_bytes"][v] = s * h * 2
        c["grad_bytes"][v] = (12 * h * h * 2) // tp
    return c


def enumerate_triples(num_devices: int, tps: Tuple[int, ...], pp_max: int) -> List[Tuple[int, int, int]]:
    """All (dp, tp, pp) with power-of-two sizes, dp*tp*pp == num_devices, pp <= pp_max."""
    out = []
    for tp in tps:
        pp = 1
        while pp <= pp_max:
            if num_devices % (tp * pp) == 0 and tp * pp <= num_devices:
                out.append((num_devices // (tp * pp), tp, pp))
            pp *= 2
    return out


def _grid(triples, m_max: int) -> Dict[str, np.ndarray]:
    dp, tp, pp, m, sc = [], [], [], [], []
    for (d, t, p) in triples:
        for mm in range(1, m_max + 1):
            for s in (0, 1):
                dp.append(d); tp.append(t); pp.append(p); m.append(mm); sc.append(s)
    n = len(dp)
    return {
        "dp": np.asarray(dp, np.int32), "tp": np.asarray(tp, np.int32),
        "pp": np.asarray(pp, np.int32), "m": np.asarray(m, np.int32),
        "schedule": np.asarray(sc, np.uint8),
        "part_off": np.full(n, -1, np.int64),
        "part_pool": np.zeros(0, np.uint8),
    }


def _uniform_bnd(L: int, pp: int) -> np.ndarray:
    return (np.arange(pp + 1, dtype=np.int64) * L) // pp


# --------------------------------------------------------------------------- workloads

def _tiny(shared_draw: bool) -> Workload:
    k = 1
    rng = _rng(k)
    L = 4
    c = _empty_costs(L, (1,))
    if shared_draw:
        f = np.full(L, rng.integers(800_000, 1_200_001), dtype=np.int64)
        b = 2 * f + rng.integers(0, 50_001)
    else:
        rng = np.random.Generator(np.random.Philox(key=BASE_SEED + k, counter=1))
        f = rng.integers(800_000, 1_200_001, size=L, dtype=np.int64)
        b = 2 * f + rng.integers(0, 50_001, size=L, dtype=np.int64)
    c["fwd_comp_ns"][0] = f
    c["bwd_comp_ns"][0] = b
    c["act_bytes"][0] = 4 * MIB
    cand = {
        "dp": np.asarray([1, 1], np.int32), "tp": np.asarray([1, 1], np.int32),
        "pp": np.asarray([2, 2], np.int32), "m": np.asarray([4, 4], np.int32),
        "schedule": np.asarray([1, 0], np.uint8),          # 1F1B first, GPipe second
        "part_off": np.asarray([0, 0], np.int64),
        "part_pool": np.asarray([0, 2, 4], np.uint8),
    }
    return Workload("tiny" if shared_draw else "tiny_b", c, _cluster(2), cand,
                    notes="4 layers, pp=2, m=4, explicit partition [0,2,4]")


def _gpt(k: int, name: str, L: int, h: int, s: int, tps, N: int, pp_cap: int, m_max: int) -> Workload:
    rng = _rng(k)
    c = _transformer_costs(rng, L, h, s, tps)
    triples = enumerate_triples(N, tps, min(pp_cap, L))
    cand = _grid(triples, m_max)
    return Workload(name, c, _cluster(N), cand, meta={"triples": triples, "rng": rng})


def _gpt96() -> Workload:
    w = _gpt(4, "gpt96", 96, 12288, 2048, (1, 2, 4, 8), 1024, 64, 512)
    rng = w.meta.pop("rng")
    w.cluster["dp_bucket_bytes"] = 25 * MIB
    L = w.L
    base = w.cand
    sel = np.nonzero(base["pp"] > 1)[0]
    reps = 3
    n_new = sel.size * reps
    tries = 32
    u = rng.random(size=(n_new, tries))
    sg = rng.integers(0, 2, size=(n_new, tries), dtype=np.int64) * 2 - 1
    pool: List[np.ndarray] = []
    offs = np.empty(n_new, np.int64)
    pos = 0
    row = 0
    for ci in sel:
        pp = int(base["pp"][ci])
        ub = _uniform_bnd(L, pp)
        for _ in range(reps):
            bnd = None
            for t in range(tries):
                b = 1 + int(u[row, t] * (pp - 1))
                nb = ub[b] + sg[row, t]
                if ub[b - 1] < nb < ub[b + 1]:
                    bnd = ub.copy()
                    bnd[b] = nb
                    break
            if bnd is None:                      # vanishingly unlikely; keep the uniform split
                bnd = ub.copy()
            pool.append(bnd.astype(np.uint8))
            offs[row] = pos
            pos += pp + 1
            row += 1
    idx = np.repeat(sel, reps)
    cand = {key: np.concatenate([base[key], base[key][idx]]) for key in ("dp", "tp", "pp", "m", "schedule")}
    cand["part_off"] = np.concatenate([base["part_off"], offs])
    cand["part_pool"] = np.concatenate(pool) if pool else np.zeros(0, np.uint8)
    w.cand = cand
    return w


def _hetero64(C: int = 1_000_000) -> Workload:
    k = 5
    rng = _rng(k)
    L, h, s = 64, 4096, 2048
    tps = (1, 2, 4, 8)
    N = 512
    scale = np.ones(L)
    moe = np.zeros(L, bool)
    moe[1::2] = True
    moe[0] = moe[L - 1] = False
    scale[moe] = 4.0
    scale[0] = scale[L - 1] = 3.0
    c = _transformer_costs(rng, L, h, s, tps, scale=scale)
    c["a2a_bytes"][:, moe] = s * h * 2
    triples = enumerate_triples(N, tps, 64)
    tri = np.asarray(triples, np.int32)
    ti = rng.integers(0, len(triples), size=C)
    m = rng.integers(1, 129, size=C).astype(np.int32)
    sc = rng.integers(0, 2, size=C).astype(np.uint8)
    pp = tri[ti, 2]
    # uniform random composition of L into pp positive parts: pp-1 distinct cuts out of L-1
    offs = np.zeros(C, np.int64)
    sizes = (pp + 1).astype(np.int64)
    offs[1:] = np.cumsum(sizes)[:-1]
    pool = np.zeros(int(sizes.sum()), np.uint8)
    for p in np.unique(pp):
        ids = np.nonzero(pp == p)[0]
        keys = rng.random(size=(ids.size, L - 1))
        cuts = np.sort(np.argsort(keys, axis=1)[:, : p - 1] + 1, axis=1)
        bnd = np.zeros((ids.size, p + 1), np.int64)
        bnd[:, 1:p] = cuts
        bnd[:, p] = L
        dst = offs[ids][:, None] + np.arange(p + 1)[None, :]
        pool[dst] = bnd.astype(np.uint8)
    cand = {
        "dp": tri[ti, 0].copy(), "tp": tri[ti, 1].copy(), "pp": pp.copy(), "m": m,
        "schedule": sc, "part_off": offs, "part_pool": pool,
    }
    return Workload("hetero64", c, _cluster(N), cand, meta={"triples": triples})


def make_workload(name: str, **kw) -> Workload:
    """Build one of CONFIG_NAMES.  ``hetero64`` accepts ``C=`` to draw a shorter list."""
    if name == "tiny":
        return _tiny(True)
    if name == "tiny_b":
        return _tiny(False)
    if name == "gpt24":
        w = _gpt(2, name, 24, 1024, 1024, (1, 2, 4, 8, 16), 16, 16, 32)
    elif name == "gpt48":
        w = _gpt(3, name, 48, 2048, 2048, (1, 2, 4, 8), 128, 32, 128)
    elif name == "gpt96":
        w = _gpt96()
    elif name == "hetero64":
        w = _hetero64(**kw)
    else:
        raise KeyError(name)
    w.meta.pop("rng", None)
    return w


def subset(w: Workload, idx) -> Workload:
    """The same tables with only the candidates ``idx`` (partition pool and explicit schedules shared,
    offsets kept)."""
    idx = np.asarray(idx, dtype=np.int64)
    shared = ("part_pool", "schedule_off", "schedule_words")
    cand = {k: (v if k in shared else v[idx].copy()) for k, v in w.cand.items()}
    return Workload(w.name + "[subset]", w.costs, dict(w.cluster), cand, w.notes, dict(w.meta))


def total_stages(w: Workload) -> int:
    return int(w.cand["pp"].astype(np.int64).sum())


# ---------------------------------------------------------------------------------------
# Inputs of the steps in front of event-flow generation (Sec. 4.1, Sec. 4.2).  No arithmetic of
# the method here: only the seeded draw of operator records and of profile records.

def make_operator_records(n: int, n_distinct: int, K: int = 6, seed: int = 2306084230 + 11) -> np.ndarray:
    """n operator records of K int64 words drawn from n_distinct distinct operators with a skewed
    (Zipf-like) popularity, the way the per-rank sub-models of one training job repeat the same
    few layer operators: word 0 an operator-name id, words 1..K-2 parameters / shape, word K-1 the
    intra-/inter-node attribute."""
    rng = np.random.Generator(np.random.Philox(seed))
    proto = rng.integers(0, 1 << 40, size=(n_distinct, K), dtype=np.int64)
    proto[:, 0] = rng.integers(0, 64, size=n_distinct)
    proto[:, K - 1] = rng.integers(0, 2, size=n_distinct)
    proto = np.unique(proto, axis=0)
    rng.shuffle(proto, axis=0)
    w = 1.0 / np.arange(1, proto.shape[0] + 1)
    pick = rng.choice(proto.shape[0], size=n, p=w / w.sum())
    return np.ascontiguousarray(proto[pick])


def make_comm_profiles(n: int, seed: int = 2306084230 + 12):
    """n communication-event profile records: kind (0 p2p, 1 all-reduce, a few invalid), ranks,
    t_a, t_b in ns."""
    rng = np.random.Generator(np.random.Philox(seed))
    kind = rng.choice(np.array([0, 1, 2], dtype=np.int32), size=n, p=[0.45, 0.54, 0.01]).astype(np.int32)
    ranks = (1 << rng.integers(0, 11, size=n)).astype(np.int32)
    odd = rng.random(n) < 0.2
    ranks[odd] = rng.integers(1, 3000, size=int(odd.sum()), dtype=np.int32)
    ranks[rng.random(n) < 0.005] = 0
    t_a = rng.integers(0, 1 << 36, size=n, dtype=np.int64)
    t_b = rng.integers(0, 1 << 36, size=n, dtype=np.int64)
    big = rng.random(n) < 0.01
    t_a[big] = rng.integers(1 << 58, 1 << 61, size=int(big.sum()), dtype=np.int64)
    t_a[rng.random(n) < 0.003] = -5
    return kind, ranks, t_a, t_b
