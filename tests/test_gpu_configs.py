"""GPU parity of tgnn_train_step at the benchmark configurations' full sizes (C1, C2, C3) and on a C4-shaped
graph: sampled neighbours and winners bit-exact on every checked step, logits / gradients / memory within
1e-4 after consecutive batches."""
import numpy as np
import pytest

from gpu_common import (GpuSide, OracleSide, batch_np, compare_state, compare_step, make_problem, rel_err,
                        spot_check_sampler)
import synth

pytestmark = pytest.mark.gpu


def run(P, n_steps, lr, check_at, first=0):
    d = P["d"]
    G = GpuSide(P); Or = OracleSide(P)
    out = {}
    for s in range(n_steps):
        lo = (first + s) * d.batch; hi = min(lo + d.batch, P["E"])
        b = batch_np(P, lo, hi)
        want = s in check_at
        # (training on: the oracle takes the GPU's ReLU decisions on every step, see OracleSide.step)
        g = G.step([b], lr=lr, want=True if want else ("gates" if lr else False))
        o = Or.step([b], lr=lr, gpu=g)
        if want:
            out[s] = compare_step(g, o, label=f"{P['name']} lr {lr} step {first + s}")
            if not Or.scan:      # the oracle read its neighbours off the index: scan the event list for sampled roots
                spot_check_sampler(P, g, [b], seed=s)
    compare_state(G.state_np(), Or.states[0], label=P["name"])
    if lr:
        for n, v in G.params.numpy().items():
            assert rel_err(v, Or.p[n]) <= 1e-4, n
    return out


def test_c1_full_size_50_batches_sgd():
    P = make_problem("C1")
    errs = run(P, 50, lr=1e-3, check_at=(0, 1, 25, 49))
    print({k: max(v.values()) for k, v in errs.items()})


def test_c1_last_ragged_batch():
    P = make_problem("C1")
    M = len(synth.batches_of(P["E"], P["d"].batch))
    run(P, 3, lr=0.0, check_at=(0, 2), first=M - 3)          # the epoch's last mini-batch has 274 events


@pytest.mark.parametrize("lr", [0.0, 1e-3])
def test_c2_static_memory_50_batches(lr):
    """The enhanced model (static + dynamic memory) on the first 100 mini-batches' worth of the C2 recipe: 50
    consecutive batches without and with SGD."""
    P = make_problem("C2", n_events=60_000)
    run(P, 50, lr=lr, check_at=(0, 1, 25, 49))


def test_c2_full_size_late_in_the_stream():
    """C2 at its full 672,447 events, four batches from event 540,000 on (long neighbour lists, 463 MB of edge
    features); the oracle reads its neighbours off the index, sampled roots are scanned."""
    P = make_problem("C2")
    run(P, 4, lr=1e-3, check_at=(0, 2, 3), first=900)


def test_c5_no_edge_features_full_size():
    """C5 (a graph without edge features, d_e = 0, with static memory; Table 2's MOOC shape) at its full 411,749
    events: 20 consecutive batches from the start with SGD, then three late in the stream."""
    P = make_problem("C5")
    run(P, 20, lr=1e-3, check_at=(0, 1, 10, 19))
    run(P, 3, lr=1e-3, check_at=(0, 2), first=600)


def test_c3_eight_replicas_time_shifted():
    P = make_problem("C3", n_events=48_000)
    d = P["d"]
    nrep = 8
    G = GpuSide(P, n_replicas=nrep); Or = OracleSide(P, n_replicas=nrep)
    spans = synth.batches_of(P["E"], d.batch)
    M = len(spans); shift = -(-M // nrep)
    for s in range(6):
        bl = [batch_np(P, *spans[(s + r * shift) % M]) for r in range(nrep)]
        g = G.step(bl, lr=1e-3)
        o = Or.step(bl, lr=1e-3, gpu=g)
        compare_step(g, o, label=f"C3 lr 1e-3 step {s}")
    for r in range(nrep):
        compare_state(G.state_np(r), Or.states[r], label=f"C3 replica {r}")
    for n, v in G.params.numpy().items():
        assert rel_err(v, Or.p[n]) <= 1e-4, n


def test_c3_replica_subset_and_order():
    P = make_problem("C3", n_events=12_000)
    d = P["d"]
    G = GpuSide(P, n_replicas=8); Or = OracleSide(P, n_replicas=8)
    spans = synth.batches_of(P["E"], d.batch)
    for s in range(3):
        reps = [5, 0, 7]                                     # any subset, any order; others stay untouched
        bl = [batch_np(P, *spans[s + 3 * i]) for i in range(3)]
        g = G.step(bl, replicas=reps)
        o = Or.step(bl, replicas=reps, gpu=g)
        compare_step(g, o, label=f"subset step {s}")
    for r in range(8):
        compare_state(G.state_np(r), Or.states[r], label=f"replica {r}")
    assert not G.state_np(3)["mem"].any()


def test_c4_shape_three_batches():
    P = make_problem("C4", n_events=400_000)
    run(P, 3, lr=0.0, check_at=(0, 2), first=90)             # start late: neighbour lists are long, memory empty
    run(P, 4, lr=0.0, check_at=(1, 3))


_C4 = {}


def c4_full():
    """The full 20,000,000-event C4 problem, built once per session: event list from the seeded host recipe, the
    14.9 GB edge-feature table drawn on the GPU (seeded) and read by the oracle through a row view, and the
    oracle's index over the event list."""
    if not _C4:
        from synth.device import HostRowView, device_normal_table
        from oracle import tgnn_oracle as O
        P = make_problem("C4", with_efeat=False)
        P["efeat"] = device_normal_table(P["E"], P["d"].d_edge, seed=synth.CONFIGS["C4"]["seed"] + 1000)
        P["efeat_host"] = HostRowView(P["efeat"])
        _C4["P"] = P
        _C4["adj"] = O.build_adjacency(P["src"], P["dst"], P["ts"], P["d"].n_nodes)
    return _C4["P"], _C4["adj"]


@pytest.mark.slow
def test_c4_full_size_fused_steps_late_in_the_stream():
    """Three consecutive fused steps of 4,000 events on the full graph from event 16,000,000 on: event ids are
    beyond 2^31 / d_e, so the edge-feature row offsets pass 2^31 elements and 2^32 bytes; neighbour lists are at
    their longest.  Indices and winners bit-exact, logits / gradients / s' of all slots / memory within 1e-4, SGD
    on."""
    P, adj = c4_full()
    d = P["d"]
    assert (16_000_000 * d.d_edge) > 2 ** 31
    G = GpuSide(P); Or = OracleSide(P)
    Or.adj = adj; Or.scan = False
    first = 4000
    for s in range(3):
        lo = (first + s) * d.batch
        b = batch_np(P, lo, lo + d.batch)
        g = G.step([b], lr=1e-3)
        o = Or.step([b], lr=1e-3, gpu=g)
        compare_step(g, o, label=f"C4 full lr 1e-3 step {first + s}")
        spot_check_sampler(P, g, [b], n=16, seed=s)
        assert g["neid"].max() > 11_600_000
    compare_state(G.state_np(), Or.states[0], label="C4 full")
    for n, v in G.params.numpy().items():
        assert rel_err(v, Or.p[n]) <= 1e-4, n


@pytest.mark.slow
def test_c4_full_graph_sampler():
    """Sampler on the full 20,000,000-event graph (node degrees up to millions) against the oracle."""
    import torch
    from paper_2307_07649_amd import tgnn
    from oracle import tgnn_oracle as O
    P, adj_full = c4_full()
    g = P
    n = synth.CONFIGS["C4"]["n_nodes"]
    ctx = tgnn.Context(n, 8, 4, 0, 0, 1, 10, 40_000)
    graph = tgnn.Graph(g["src"], g["dst"], g["ts"], n, None)
    rng = np.random.default_rng(0)
    Q = 100_000
    ev = rng.integers(0, len(g["src"]), Q)
    qn = np.where(rng.random(Q) < 0.5, g["src"][ev], g["dst"][ev]).astype(np.int32)
    qt = g["ts"][ev].copy()
    qt[::7] = rng.uniform(0, 1.4e5, len(qt[::7]))
    nbr, eid, ts, cnt = ctx.tgnn_sample_recent(graph, torch.from_numpy(qn).cuda(), torch.from_numpy(qt).cuda())
    o = O.sample_recent_indexed(adj_full, qn, qt, 10)
    assert np.array_equal(cnt.cpu().numpy(), o[3]) and np.array_equal(eid.cpu().numpy(), o[1])
    assert np.array_equal(nbr.cpu().numpy(), o[0]) and np.array_equal(ts.cpu().numpy(), o[2])
    pick = rng.choice(Q, 24, replace=False)               # the scan of the whole event list for sampled queries
    sc = O.sample_recent(g["src"], g["dst"], g["ts"], qn[pick], qt[pick], 10)
    for a, b in zip(sc, o):
        assert np.array_equal(a, b[pick])


def test_c1_and_c3_four_steps_per_call():
    """tgnn_train_steps at the benchmark's sizes, in the launch configuration bench.py times (groups of four steps,
    SGD, gradients cleared inside the step): C1 for 12 batches and C3's eight replicas for 4 steps, against the
    oracle stepping one step at a time: every step's loss, the final memory and mails, the final parameters."""
    import torch
    from paper_2307_07649_amd import tgnn
    for name, n_ev, nrep, n_steps in (("C1", None, 1, 12), ("C3", 48_000, 8, 4)):
        P = make_problem(name, n_events=n_ev)
        d = P["d"]
        G = GpuSide(P, n_replicas=nrep, flags=tgnn.FLAG_OVERWRITE_GRADS); Or = OracleSide(P, n_replicas=nrep)
        spans = synth.batches_of(P["E"], d.batch)
        M = len(spans); shift = -(-M // nrep)
        losses = torch.zeros(4, device="cuda")
        g_loss, o_loss = [], []
        with torch.cuda.stream(G.stream):
            for s0 in range(0, n_steps, 4):
                steps = []
                for s in range(s0, s0 + 4):
                    bl = [batch_np(P, *spans[(s + r * shift) % M]) for r in range(nrep)]
                    steps.append([tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"], replica=r) for r, b in enumerate(bl)])
                    o_loss.append(Or.step(bl, lr=1e-3)["loss"])
                G.ctx.tgnn_train_steps(G.graph, G.state, G.params, G.grads, steps, lr=1e-3, out_loss=losses)
                torch.cuda.synchronize()
                g_loss += [float(x) for x in losses.cpu().numpy()]
        for s, (a, b) in enumerate(zip(g_loss, o_loss)):
            assert abs(a - b) <= 1e-4 * abs(b), (name, s, a, b)
        for r in range(nrep):
            compare_state(G.state_np(r), Or.states[r], label=f"{name} replica {r}")
        for n, v in G.params.numpy().items():
            assert rel_err(v, Or.p[n]) <= 1e-4, (name, n)
