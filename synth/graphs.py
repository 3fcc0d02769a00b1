"""Synthetic temporal graphs shaped like the paper's workloads (Table 2 gives |V|, |E|,
max(t) and feature widths; the experiment section gives d_mem = 100, k = 10 and local
batch sizes 600 / 3200).  The real datasets are not available, so seeded random graphs
with the same shapes stand in for them.

Everything here is input generation: numpy random draws and array layout only.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np


@dataclass(frozen=True)
class ModelDims:
    n_nodes: int
    d_mem: int
    d_time: int
    d_edge: int
    d_static: int
    n_heads: int
    k: int
    batch: int
    n_replicas: int = 1
    n_classes: int = 0     # > 0: edge classification with that many outputs instead of link prediction

    @property
    def d_in(self):        # GRU input: mail (2 d_mem) | time encoding | edge feature
        return 2 * self.d_mem + self.d_time + self.d_edge

    @property
    def d_x(self):         # node input of the attention layer: dynamic | static memory
        return self.d_mem + self.d_static

    @property
    def d_q(self):
        return self.d_x + self.d_time

    @property
    def d_kv(self):
        return self.d_x + self.d_edge + self.d_time

    @property
    def d_out(self):
        return self.d_mem


# name -> generator recipe.  "src_range"/"dst_range" are half-open id ranges.
CONFIGS = {
    "C0": dict(seed=0, n_nodes=1000, n_events=20_000, kind="uniform", ts="int_steps",
               d_mem=32, d_time=32, d_edge=16, d_static=0, n_heads=1, k=10, batch=200,
               n_replicas=1, neg_range=(0, 1000)),
    "C1": dict(seed=1, n_nodes=9227, n_events=157_474, kind="bipartite_zipf",
               n_src=8227, n_dst=1000, zipf_src=1.2, zipf_dst=1.5, ts="uniform", t_max=2.7e6,
               d_mem=100, d_time=100, d_edge=172, d_static=0, n_heads=2, k=10, batch=600,
               n_replicas=1, neg_range=(8227, 9227)),
    "C2": dict(seed=2, n_nodes=10_984, n_events=672_447, kind="bipartite_zipf",
               n_src=10_000, n_dst=984, zipf_src=1.1, zipf_dst=1.3, ts="uniform", t_max=2.7e6,
               d_mem=100, d_time=100, d_edge=172, d_static=100, n_heads=2, k=10, batch=600,
               n_replicas=1, neg_range=(10_000, 10_984)),
    "C3": dict(seed=2, n_nodes=10_984, n_events=672_447, kind="bipartite_zipf",
               n_src=10_000, n_dst=984, zipf_src=1.1, zipf_dst=1.3, ts="uniform", t_max=2.7e6,
               d_mem=100, d_time=100, d_edge=172, d_static=100, n_heads=2, k=10, batch=600,
               n_replicas=8, neg_range=(10_000, 10_984)),
    # no edge features (Table 2: MOOC, 7,144 nodes = 7,047 users + 97 course items, 411,749 events, max(t) 2.6e7,
    # pre-trained static node features of width 100)
    "C5": dict(seed=5, n_nodes=7144, n_events=411_749, kind="bipartite_zipf",
               n_src=7047, n_dst=97, zipf_src=0.9, zipf_dst=1.0, ts="uniform", t_max=2.6e7,
               d_mem=100, d_time=100, d_edge=0, d_static=100, n_heads=2, k=10, batch=600,
               n_replicas=1, neg_range=(7047, 7144)),
    "C4": dict(seed=4, n_nodes=16_682, n_events=20_000_000, kind="zipf", zipf=1.05,
               ts="bursty", t_max=1.4e5,
               d_mem=100, d_time=100, d_edge=186, d_static=0, n_heads=2, k=10, batch=4000,
               n_replicas=1, neg_range=(0, 16_682)),
}


def dims_of(name: str, **override) -> ModelDims:
    c = dict(CONFIGS[name]); c.update(override)
    return ModelDims(n_nodes=c["n_nodes"], d_mem=c["d_mem"], d_time=c["d_time"], d_edge=c["d_edge"],
                     d_static=c["d_static"], n_heads=c["n_heads"], k=c["k"], batch=c["batch"],
                     n_replicas=c["n_replicas"], n_classes=c.get("n_classes", 0))


def _zipf_ids(rng, n_ids, a, size, lo=0):
    """ids in [lo, lo+n_ids) with probability proportional to rank^-a under a random rank->id map."""
    p = np.arange(1, n_ids + 1, dtype=np.float64) ** (-a)
    cdf = np.cumsum(p); cdf /= cdf[-1]
    ranks = np.searchsorted(cdf, rng.random(size), side="left").astype(np.int64)
    np.minimum(ranks, n_ids - 1, out=ranks)
    perm = rng.permutation(n_ids)
    return (perm[ranks] + lo).astype(np.int32)


def gen_graph(name: str, n_events: int | None = None, with_efeat: bool = True, efeat_chunk: int = 1 << 20):
    """Return dict(src, dst, ts, efeat) for config `name`.

    src, dst: int32 [E]; ts: float64 [E] non-decreasing; efeat: float32 [E, d_edge] ~ N(0,1).
    `n_events` shortens the event list (same recipe, fewer draws) for tests.
    """
    c = CONFIGS[name]
    E = int(n_events if n_events is not None else c["n_events"])
    rng = np.random.Generator(np.random.PCG64(c["seed"]))
    kind = c["kind"]
    if kind == "uniform":
        n = c["n_nodes"]
        src = rng.integers(0, n, E, dtype=np.int64)
        dst = rng.integers(0, n - 1, E, dtype=np.int64)
        dst = np.where(dst >= src, dst + 1, dst)                # src != dst, still uniform
        src, dst = src.astype(np.int32), dst.astype(np.int32)
    elif kind == "bipartite_zipf":
        src = _zipf_ids(rng, c["n_src"], c["zipf_src"], E, 0)
        dst = _zipf_ids(rng, c["n_dst"], c["zipf_dst"], E, c["n_src"])
    elif kind == "zipf":
        n = c["n_nodes"]
        src = _zipf_ids(rng, n, c["zipf"], E, 0)
        dst = _zipf_ids(rng, n, c["zipf"], E, 0)
        for _ in range(64):                                      # redraw self-loops
            bad = np.nonzero(src == dst)[0]
            if bad.size == 0:
                break
            dst[bad] = rng.integers(0, n, bad.size, dtype=np.int64).astype(np.int32)
        assert not np.any(src == dst)
    else:
        raise ValueError(kind)

    if c["ts"] == "int_steps":
        ts = np.cumsum(rng.integers(1, 6, E, dtype=np.int64)).astype(np.float64)
        ts -= ts[0]
    elif c["ts"] == "uniform":
        ts = np.sort(rng.random(E) * c["t_max"])
    elif c["ts"] == "bursty":
        flips = rng.random(E) < 1e-3
        state = (np.cumsum(flips) & 1).astype(bool)
        gaps = rng.standard_exponential(E) * np.where(state, 0.1, 10.0)
        ts = np.cumsum(gaps)
        ts *= c["t_max"] / ts[-1]
    else:
        raise ValueError(c["ts"])

    out = dict(src=src, dst=dst, ts=np.ascontiguousarray(ts, dtype=np.float64))
    if with_efeat:
        d_e = c["d_edge"]
        frng = np.random.Generator(np.random.PCG64(c["seed"] + 1000))
        ef = np.empty((E, d_e), dtype=np.float32)
        for lo in range(0, E, efeat_chunk):
            hi = min(E, lo + efeat_chunk)
            ef[lo:hi] = frng.standard_normal((hi - lo, d_e), dtype=np.float32)
        out["efeat"] = ef
    return out


def gen_negatives(name: str, n_events: int, group: int = 0):
    """One negative destination per event, uniform over the config's destination id range.
    The paper pre-samples a few groups of negatives offline and reuses them; `group` selects one."""
    c = CONFIGS[name]
    lo, hi = c["neg_range"]
    rng = np.random.Generator(np.random.PCG64(c["seed"] + 2000 + group))
    return rng.integers(lo, hi, n_events, dtype=np.int64).astype(np.int32)


def gen_labels(n_events: int, n_classes: int, n_true: int, seed: int = 0):
    """Multi-label targets of an edge-classification task, float32 [E, C] in {0, 1}: every event has `n_true`
    distinct true classes (the GDELT task of Sec. 4 has 56 classes, 6 of them true), drawn with a skewed class
    popularity (probability proportional to 1 / (1 + class index))."""
    rng = np.random.Generator(np.random.PCG64(seed + 5000))
    w = 1.0 / (1.0 + np.arange(n_classes))
    # n_true distinct classes per event: the largest of exponential races (Gumbel top-k)
    keys = np.log(w)[None, :] + rng.gumbel(size=(n_events, n_classes))
    top = np.argpartition(-keys, n_true - 1, axis=1)[:, :n_true]
    y = np.zeros((n_events, n_classes), np.float32)
    np.put_along_axis(y, top, 1.0, axis=1)
    return y


def gen_static(name: str):
    """Frozen static node memory, N(0, 0.1), float32 [n_nodes, d_static]; None when d_static == 0."""
    c = CONFIGS[name]
    if c["d_static"] == 0:
        return None
    rng = np.random.Generator(np.random.PCG64(c["seed"] + 3000))
    return (0.1 * rng.standard_normal((c["n_nodes"], c["d_static"]))).astype(np.float32)


PARAM_SHAPES = lambda d: {  # noqa: E731  (name -> (shape, fan_in))
    "gru_wih": ((3 * d.d_mem, d.d_in), d.d_in), "gru_whh": ((3 * d.d_mem, d.d_mem), d.d_mem),
    "gru_bih": ((3 * d.d_mem,), d.d_in), "gru_bhh": ((3 * d.d_mem,), d.d_mem),
    "wq": ((d.d_out, d.d_q), d.d_q), "bq": ((d.d_out,), d.d_q),
    "wk": ((d.d_out, d.d_kv), d.d_kv), "bk": ((d.d_out,), d.d_kv),
    "wv": ((d.d_out, d.d_kv), d.d_kv), "bv": ((d.d_out,), d.d_kv),
    "wo": ((d.d_out, d.d_out + d.d_x), d.d_out + d.d_x), "bo": ((d.d_out,), d.d_out + d.d_x),
    "dec_ws": ((d.d_out, d.d_out), d.d_out), "dec_wd": ((d.d_out, d.d_out), d.d_out),
    "dec_b1": ((d.d_out,), d.d_out),
    "dec_w2": (((d.n_classes, d.d_out) if d.n_classes else (d.d_out,)), d.d_out),
    "dec_b2": ((d.n_classes if d.n_classes else 1,), d.d_out),
}

PARAM_ORDER = ["time_w", "time_b", "gru_wih", "gru_whh", "gru_bih", "gru_bhh", "wq", "bq", "wk", "bk",
               "wv", "bv", "wo", "bo", "dec_ws", "dec_wd", "dec_b1", "dec_w2", "dec_b2"]


def gen_params(d: ModelDims, seed: int = 0, random_phase: bool = False):
    """Initial weights, float32: uniform(-1/sqrt(fan_in), 1/sqrt(fan_in)) for every matrix and bias.
    Time-encoding frequencies w_c = 10^(-9 c / (d_time - 1)) and phases 0 (or uniform(-pi, pi))."""
    rng = np.random.Generator(np.random.PCG64(seed + 4000))
    p = {}
    c = np.arange(d.d_time, dtype=np.float64)
    p["time_w"] = (10.0 ** (-9.0 * c / max(d.d_time - 1, 1))).astype(np.float32)
    p["time_b"] = (rng.uniform(-np.pi, np.pi, d.d_time).astype(np.float32) if random_phase
                   else np.zeros(d.d_time, dtype=np.float32))
    for name, (shape, fan_in) in PARAM_SHAPES(d).items():
        b = 1.0 / np.sqrt(fan_in)
        p[name] = rng.uniform(-b, b, shape).astype(np.float32)
    return {k: p[k] for k in PARAM_ORDER}


def batches_of(n_events: int, batch: int):
    """[(lo, hi)] consecutive chronological mini-batches; the last one may be short."""
    return [(lo, min(lo + batch, n_events)) for lo in range(0, n_events, batch)]
