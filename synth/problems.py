"""One problem = one seeded synthetic workload: event list, edge features, negative destinations, static
memory, initial weights and the model widths.  Input generation only (random draws and array layout)."""
from __future__ import annotations

import numpy as np

from .graphs import CONFIGS, ModelDims, dims_of, gen_graph, gen_labels, gen_negatives, gen_params, gen_static


def make_problem(name, n_events=None, random_phase=False, with_efeat=True, with_labels=True, **dims_override):
    """The benchmark configuration `name` (C0..C4), optionally with a shortened event list (same recipe, fewer
    draws).  with_efeat=False leaves the edge-feature table out (the caller fills P["efeat"] itself), with_labels=False
    the class targets of an edge-classification variant."""
    g = gen_graph(name, n_events=n_events, with_efeat=with_efeat)
    d = dims_of(name, **dims_override)
    E = len(g["src"])
    P = dict(name=name, d=d, src=g["src"], dst=g["dst"], ts=g["ts"], efeat=g.get("efeat"), E=E,
             neg=gen_negatives(name, E), static=gen_static(name),
             params=gen_params(d, seed=CONFIGS[name]["seed"], random_phase=random_phase))
    if d.n_classes and with_labels:     # (n_classes=C as an override: the same graph as an edge-classification task)
        P["labels"] = gen_labels(E, d.n_classes, min(6, d.n_classes), seed=CONFIGS[name]["seed"])
    return P


def custom_problem(n_nodes, E, d_mem, d_time, d_edge, d_static, n_heads, k, batch, seed=0, tmax=100.0, ties=False,
                   self_loops=0.0, neg_is_dst=0.0, n_classes=0, n_true=1):
    """A small random problem of any shape.  ties: integer timestamps (many equal); self_loops / neg_is_dst:
    fraction of events whose destination is their source / whose negative destination is their true one;
    n_classes > 0: an edge-classification problem with n_true true classes per event (P["labels"])."""
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n_nodes, E).astype(np.int32)
    dst = ((src + rng.integers(1, n_nodes, E)) % n_nodes).astype(np.int32)
    ts = np.sort(rng.integers(0, int(tmax), E).astype(np.float64)) if ties else np.sort(rng.uniform(0, tmax, E))
    d = ModelDims(n_nodes=n_nodes, d_mem=d_mem, d_time=d_time, d_edge=d_edge, d_static=d_static,
                  n_heads=n_heads, k=k, batch=batch, n_classes=n_classes)
    efeat = rng.standard_normal((E, d_edge)).astype(np.float32)
    neg = rng.integers(0, n_nodes, E).astype(np.int32)
    static = (0.1 * rng.standard_normal((n_nodes, d_static))).astype(np.float32) if d_static else None
    if self_loops > 0.0:
        loop = rng.random(E) < self_loops
        dst = np.where(loop, src, dst).astype(np.int32)
    if neg_is_dst > 0.0:
        same = rng.random(E) < neg_is_dst
        neg = np.where(same, dst, neg).astype(np.int32)
    P = dict(name="custom", d=d, src=src, dst=dst, ts=ts, E=E, efeat=efeat, neg=neg, static=static,
             params=gen_params(d, seed=seed, random_phase=True))
    if n_classes:
        P["labels"] = gen_labels(E, n_classes, n_true, seed=seed)
    return P


def batch_np(P, lo, hi):
    """Events lo .. hi - 1 of problem P as one chronological mini-batch (host arrays)."""
    b = dict(src=P["src"][lo:hi], dst=P["dst"][lo:hi], neg=P["neg"][lo:hi],
             eid=np.arange(lo, hi, dtype=np.int32), t=P["ts"][lo:hi])
    if P.get("labels") is not None:
        b["labels"] = P["labels"][lo:hi]
    return b
