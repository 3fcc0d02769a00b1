"""GPU parity of the fused training step (tgnn_train_step through the C ABI) against the CPU oracle on
the same seeded inputs: bit-exact sampled neighbours and write-back winners, 1e-4 relative on logits,
gradients and the memory after 50 consecutive batches."""
import numpy as np
import pytest

from gpu_common import GpuSide, OracleSide, batch_np, compare_state, compare_step, custom_problem, make_problem

pytestmark = pytest.mark.gpu


def run_sequence(P, n_steps, lr=0.0, check_at=(0,), dt_source=0, first=0, own_stream=True, flags=0):
    d = P["d"]
    G = GpuSide(P, dt_source=dt_source, own_stream=own_stream, flags=flags); Or = OracleSide(P, dt_source=dt_source)
    errs = {}
    for s in range(n_steps):
        lo = (first + s) * d.batch; hi = min(lo + d.batch, P["E"])
        b = batch_np(P, lo, hi)
        want = s in check_at or s == n_steps - 1
        # with training on, the oracle takes the GPU's ReLU decisions on EVERY step: a tie gated the other way on an
        # unchecked step would send the two parameter trajectories apart by a whole gradient term times lr
        g = G.step([b], lr=lr, want=True if want else ("gates" if lr else False))
        o = Or.step([b], lr=lr, gpu=g)
        if want:
            errs[s] = compare_step(g, o, label=f"step {s}")
    e = compare_state(G.state_np(), Or.states[0], label="state")
    if lr:
        from gpu_common import rel_err
        for n, v in G.params.numpy().items():
            assert rel_err(v, Or.p[n]) <= 1e-4, n
    return errs, e


def test_c0_50_batches_lr0():
    P = make_problem("C0", random_phase=True)
    errs, e = run_sequence(P, 50, lr=0.0, check_at=(0, 1, 10, 49))
    print(errs[49], e)


def test_c0_50_batches_sgd():
    P = make_problem("C0", random_phase=True)
    run_sequence(P, 50, lr=0.05, check_at=(0, 49))


def test_c0_edge_time_variant():
    P = make_problem("C0")
    run_sequence(P, 12, check_at=(0, 11), dt_source=1)


@pytest.mark.parametrize("own_stream,flags", [(False, 0), (True, 2), (True, 4), (True, 6), (True, 8), (True, 16)])
def test_launch_modes_agree_with_the_oracle(own_stream, flags):
    """NULL stream (direct launches); captured graph with the side stream; no graph; no graph with the side stream;
    16 events per workgroup in the root chain (small steps take 5 by default); the attention kernels' generic code
    path on a shape that fits their register-resident one.
    (The default, a captured single-stream graph, is what every other test runs.)"""
    P = make_problem("C0", random_phase=True)
    run_sequence(P, 12, lr=0.05, check_at=(0, 5, 11), own_stream=own_stream, flags=flags)


@pytest.mark.parametrize("shape", [
    dict(n_nodes=50, E=600, d_mem=8, d_time=4, d_edge=3, d_static=2, n_heads=2, k=3, batch=37),     # nothing aligned
    dict(n_nodes=40, E=900, d_mem=24, d_time=10, d_edge=0, d_static=0, n_heads=3, k=10, batch=100, ties=True),
    dict(n_nodes=300, E=800, d_mem=100, d_time=100, d_edge=186, d_static=0, n_heads=2, k=10, batch=64),
    dict(n_nodes=64, E=640, d_mem=32, d_time=16, d_edge=8, d_static=12, n_heads=4, k=32, batch=64),
    # widths the one-launch root chain does not take (not a multiple of 4; wider than 128): separate launches
    dict(n_nodes=45, E=400, d_mem=18, d_time=6, d_edge=5, d_static=0, n_heads=3, k=4, batch=41),
    dict(n_nodes=60, E=300, d_mem=132, d_time=12, d_edge=7, d_static=0, n_heads=2, k=5, batch=50),
    # the root chain at its widest (8 column blocks), ragged 16-event tiles
    dict(n_nodes=60, E=300, d_mem=128, d_time=12, d_edge=7, d_static=3, n_heads=4, k=5, batch=50),
    # slot inputs wider than the attention kernels keep in registers (d_e > 192, d_t > 128), two heads, k = 10
    dict(n_nodes=80, E=600, d_mem=32, d_time=130, d_edge=200, d_static=0, n_heads=2, k=10, batch=60),
    # the register-resident attention path at its limits: d_e = 192, d_t = 128, d_o = 128, one head
    dict(n_nodes=80, E=600, d_mem=128, d_time=128, d_edge=192, d_static=0, n_heads=1, k=10, batch=60),
])
def test_odd_shapes(shape):
    P = custom_problem(**shape)
    n = P["E"] // P["d"].batch
    run_sequence(P, min(n, 8), check_at=(0, 3))


def test_self_loop_events_and_negative_equal_to_the_true_destination():
    """A quarter of the events have destination = source (the node is listed twice in its own neighbour list, and
    of the two occurrences in the event the destination one wins the write-back, its mail holding its own s' twice);
    a quarter of the negative destinations are the true destination."""
    P = custom_problem(n_nodes=40, E=1200, d_mem=32, d_time=16, d_edge=8, d_static=4, n_heads=2, k=6, batch=100,
                       self_loops=0.25, neg_is_dst=0.25)
    assert (P["src"] == P["dst"]).sum() > 100 and (P["neg"] == P["dst"]).sum() > 100
    errs, _ = run_sequence(P, 12, lr=0.02, check_at=(0, 1, 5, 11))
    # 16 events per workgroup in the root chain as well
    run_sequence(P, 6, lr=0.0, check_at=(0, 5), flags=8)


def test_ragged_last_batch_and_single_event():
    P = custom_problem(n_nodes=30, E=205, d_mem=16, d_time=8, d_edge=4, d_static=0, n_heads=2, k=5, batch=50)
    run_sequence(P, 5, check_at=(0, 4))      # last batch has 5 events
    P = custom_problem(n_nodes=30, E=40, d_mem=16, d_time=8, d_edge=4, d_static=0, n_heads=2, k=5, batch=1)
    run_sequence(P, 40, check_at=(0, 39))


def test_sampled_stage_timing_and_row_count():
    """Stage timing on every 4th step (tgnn_profile_every): the timed steps are launched kernel by kernel, the others
    replay the captured graph; both agree with the oracle, the record holds exactly the timed steps, and the
    distinct-row count the step leaves behind (debug item 8) is the number of distinct nodes among the roots and
    their sampled neighbours."""
    import torch
    P = make_problem("C0", random_phase=True)
    d = P["d"]
    G = GpuSide(P); Or = OracleSide(P)
    G.ctx.tgnn_profile_enable((1 << 8) | (1 << 18))
    G.ctx.tgnn_profile_every(4)
    for s in range(9):                        # timed: steps 0, 4, 8
        b = batch_np(P, s * d.batch, (s + 1) * d.batch)
        g = G.step([b], lr=0.05, want=True)
        o = Or.step([b], lr=0.05, gpu=g)
        compare_step(g, o, label=f"step {s}")
        out = o["outs"][0]
        roots = np.concatenate([b["src"], b["dst"], b["neg"]])
        nbr = out["nbr"][out["nbr"] >= 0]
        rows = torch.zeros(1, dtype=torch.int32, device="cuda")
        G.ctx.tgnn_debug_read(8, rows)
        assert int(rows.item()) == len(np.unique(np.concatenate([roots, nbr]))), s
    n_kv, ms_kv = G.ctx.tgnn_profile_read(8)
    n_empty, ms_empty = G.ctx.tgnn_profile_read(18)
    assert n_kv == 3 and n_empty == 3 and ms_kv > 0.0 and ms_empty >= 0.0
    G.ctx.tgnn_profile_enable(0)
    G.ctx.tgnn_profile_every(1)
    compare_state(G.state_np(), Or.states[0], label="state")


@pytest.mark.parametrize("per_call,flags", [(4, 0), (3, 0), (8, 0), (4, 4)])
def test_several_steps_per_call_agree_with_the_oracle(per_call, flags):
    """tgnn_train_steps: groups of consecutive steps in one call (one recorded graph per group shape; flags = 4:
    no graph, the steps are issued one by one inside the call), with SGD, against the oracle stepping one batch at a
    time: the loss of every step, the memory, mails and parameters at the end.  24 batches of C0 end with a ragged
    group when per_call does not divide them (3 -> whole groups, 8 -> whole groups, 4 -> whole groups; the last batch
    of the sequence is shorter, so its group falls back to single steps)."""
    import torch
    from paper_2307_07649_amd import tgnn
    from gpu_common import rel_err
    P = make_problem("C0", random_phase=True)
    d = P["d"]
    n_total = 24
    first = P["E"] // d.batch - n_total + 1          # the sequence ends with the ragged last batch of the graph
    G = GpuSide(P, flags=flags | tgnn.FLAG_OVERWRITE_GRADS); Or = OracleSide(P)
    spans = [((first + s) * d.batch, min((first + s + 1) * d.batch, P["E"])) for s in range(n_total)]
    assert spans[-1][1] - spans[-1][0] < d.batch
    o_loss = []
    g_loss = []
    losses = torch.zeros(per_call, device="cuda")
    with torch.cuda.stream(G.stream):
        for s0 in range(0, n_total, per_call):
            grp = spans[s0:s0 + per_call]
            steps = []
            for lo, hi in grp:
                b = batch_np(P, lo, hi)
                steps.append([tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"])])
                o_loss.append(Or.step([b], lr=0.05)["loss"])
            G.ctx.tgnn_train_steps(G.graph, G.state, G.params, G.grads, steps, lr=0.05, out_loss=losses)
            torch.cuda.synchronize()
            g_loss += [float(x) for x in losses[:len(grp)].cpu().numpy()]
    assert len(g_loss) == n_total
    for s, (a, b) in enumerate(zip(g_loss, o_loss)):
        assert abs(a - b) <= 1e-4 * max(abs(b), 1e-30), (s, a, b)
    compare_state(G.state_np(), Or.states[0], label="state")
    for n, v in G.params.numpy().items():
        assert rel_err(v, Or.p[n]) <= 1e-4, n


def test_node_ids_outside_the_range_are_counted_and_never_written():
    """Batch node ids live on the device, where the host cannot validate them: an id outside [0, n_nodes) is computed
    as node 0, wins no write-back, and is counted (tgnn_debug_read item 9); the rest of the step is unaffected in the
    sense that every other occurrence is arbitrated and written as usual."""
    import torch
    P = custom_problem(n_nodes=50, E=300, d_mem=16, d_time=8, d_edge=4, d_static=0, n_heads=2, k=5, batch=60)
    d = P["d"]
    G = GpuSide(P)
    for s in range(2):
        G.step([batch_np(P, s * 60, (s + 1) * 60)], want=False)
    b = {k_: v.copy() for k_, v in batch_np(P, 120, 180).items()}
    b["src"][3] = d.n_nodes + 5; b["dst"][7] = -2; b["neg"][1] = 10 ** 6; b["dst"][11] = d.n_nodes
    before = G.state_np()
    g = G.step([b])
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    G.ctx.tgnn_debug_read(9, cnt)
    assert int(cnt.item()) == 4
    assert np.isfinite(g["loss"]) and np.all(np.isfinite(g["logits"]))
    win = g["winner"]                                   # [src occurrences | dst occurrences]
    assert win[3] == 0 and win[60 + 7] == 0 and win[60 + 11] == 0
    after = G.state_np()
    valid = np.concatenate([np.delete(b["src"], 3), np.delete(b["dst"], [7, 11])])
    touched = np.zeros(d.n_nodes, bool); touched[valid] = True
    assert win.sum() == touched.sum()
    for name in before:
        assert np.array_equal(before[name][~touched], after[name][~touched]), name
    assert np.all(after["mail_eid"][touched] >= 120)


@pytest.mark.parametrize("J,shape", [
    (3, dict(n_nodes=60, E=900, d_mem=32, d_time=16, d_edge=8, d_static=4, n_heads=2, k=6, batch=100)),
    (2, dict(n_nodes=300, E=1600, d_mem=100, d_time=100, d_edge=172, d_static=0, n_heads=2, k=10, batch=200)),
    (8, dict(n_nodes=40, E=300, d_mem=18, d_time=6, d_edge=5, d_static=0, n_heads=3, k=4, batch=41)),
])
def test_epoch_parallel_step_against_the_oracle(J, shape):
    """tgnn_train_step_epoch_parallel (Sec. 3.2.2): J negative sets per positive batch in one step, the positive roots'
    inputs and embeddings shared, memory written once.  Against the oracle's step with the same J sets: indices and
    winners bit-exact, logits of all (1 + J) n pairs, gradients, s' of all slots, memory and parameters within 1e-4."""
    from gpu_common import rel_err
    P = custom_problem(**shape)
    d = P["d"]
    rng = np.random.default_rng(5)
    G = GpuSide(P, max_neg_sets=J); Or = OracleSide(P)
    n_steps = min(P["E"] // d.batch, 7)
    for s in range(n_steps):
        b = batch_np(P, s * d.batch, (s + 1) * d.batch)
        b["neg"] = rng.integers(0, d.n_nodes, (J, d.batch)).astype(np.int32)
        g = G.step([b], lr=0.02, n_neg_sets=J)
        o = Or.step([b], lr=0.02, gpu=g)
        compare_step(g, o, label=f"epoch-parallel J={J} step {s}")
    compare_state(G.state_np(), Or.states[0], label="state")
    for n, v in G.params.numpy().items():
        assert rel_err(v, Or.p[n]) <= 1e-4, n
    # one set through the same entry point is the plain step
    G1 = GpuSide(P, max_neg_sets=J); G2 = GpuSide(P)
    b = batch_np(P, 0, d.batch)
    a1 = G1.step([b], n_neg_sets=1); a2 = G2.step([b])
    assert np.array_equal(a1["logits"], a2["logits"]) and np.array_equal(a1["winner"], a2["winner"])


def test_adam_50_batches_against_the_oracle():
    """Adam in the step's last launch (tgnn_set_optimizer), two checks.
    (1) The optimiser's arithmetic alone, on the checked steps: the oracle's Adam, given the GPU's own parameters,
    moments and gradients of that step, reproduces the GPU's new parameters and moments to 1e-6 of each tensor's scale.
    (2) 50 consecutive C0 batches, each side on its own trajectory.  Adam divides by sqrt(v): where an element's
    gradient is small against its tensor's largest, a gradient error delta that the 1e-4-of-the-tensor's-scale rule
    admits moves the update m^/(sqrt(v^) + eps) by up to 2 delta / (sqrt(v^) - delta) (m^ moves by at most delta, so does
    sqrt(v^), and |m^| <= sqrt(v^) up to the bias corrections), at most by 2.  A parameter element is therefore held to
    1e-4 of its tensor's scale plus lr times that bound summed over the steps, with delta = 1e-4 max|g| of the step, the
    largest so far, and sqrt(v^) from the oracle; the moments themselves are linear (m) and quadratic (v) in the
    gradients and are held to 1e-4 and 2e-4.  The key bias is the limiting case: its exact gradient is zero (the
    softmax is invariant to a shift of a root's scores), both sides hold rounding noise there and the bound is 2 lr
    per step.  Frequencies and phases stay frozen."""
    import torch
    from gpu_common import rel_err, ERR_LOG
    from paper_2307_07649_amd import tgnn
    from oracle import tgnn_oracle as O
    P = make_problem("C0", random_phase=True)
    d = P["d"]
    G = GpuSide(P); Or = OracleSide(P)
    m = tgnn.Params.zeros_like(G.params); v = tgnn.Params.zeros_like(G.params)
    b1, b2, eps = (float(np.float32(x)) for x in (0.9, 0.999, 1e-8))    # the entry point takes them as fp32
    G.ctx.tgnn_set_optimizer(1, m, v, b1, b2, eps)
    Or.use_adam(b1, b2, eps)
    lr = 1e-3
    n_steps = 50
    slack = {n: np.zeros_like(x, dtype=np.float64) for n, x in Or.p.items()}
    delta = {n: 0.0 for n in Or.p}
    for s in range(n_steps):
        b = batch_np(P, s * d.batch, (s + 1) * d.batch)
        want = s in (0, 1, 25, 49)
        if want:
            before = (G.params.numpy(), m.numpy(), v.numpy())
        g = G.step([b], lr=lr, want=True if want else "gates")     # (the GPU's ReLU decisions on every step)
        o = Or.step([b], lr=lr, gpu=g)
        for n in slack:
            if n in O.FROZEN_IN_SGD:
                continue
            delta[n] = max(delta[n], 1e-4 * float(np.abs(o["grads"][n]).max()))
            root_v = np.sqrt(Or.adam_state["v"][n] / (1.0 - b2 ** (s + 1)))
            slack[n] += lr * np.minimum(2.0, 2.0 * delta[n] / np.maximum(root_v - delta[n], 1e-300))
        if want:
            compare_step(g, o, label=f"adam step {s}")
            # (1): one update from the GPU's own state and gradients
            p1 = {n: x.astype(np.float64) for n, x in before[0].items()}
            st = dict(m={n: x.astype(np.float64) for n, x in before[1].items()},
                      v={n: x.astype(np.float64) for n, x in before[2].items()}, t=s)
            O.adam(p1, {n: x.astype(np.float64) for n, x in g["grads"].items()}, st, lr, b1, b2, eps)
            after = (G.params.numpy(), m.numpy(), v.numpy())
            for n in p1:
                assert rel_err(after[0][n], p1[n]) <= 1e-6, ("update", s, n)
                assert rel_err(after[1][n], st["m"][n]) <= 1e-6, ("m update", s, n)
                assert rel_err(after[2][n], st["v"][n]) <= 1e-6, ("v update", s, n)
    compare_state(G.state_np(), Or.states[0], label="adam state")
    gp, gm, gv = G.params.numpy(), m.numpy(), v.numpy()
    traj = {}
    for n in gp:
        dev = np.abs(gp[n] - Or.p[n])
        scale = float(np.abs(Or.p[n]).max())
        traj[n] = float(dev.max()) / max(scale, 1e-30)
        assert np.all(dev <= 1e-4 * scale + slack[n]), (n, float(dev.max()) / scale)
        if n not in ("time_w", "time_b", "bk"):     # (bk: both sides hold noise only)
            assert rel_err(gm[n], Or.adam_state["m"][n]) <= 1e-4, ("m", n)
            assert rel_err(gv[n], Or.adam_state["v"][n]) <= 2e-4, ("v", n)        # v is quadratic in the gradient
    ERR_LOG.append(("adam parameters after 50 steps", traj))
    assert np.array_equal(gp["time_w"], P["params"]["time_w"]) and not gm["time_w"].any()
    # moved by about n_steps * lr, i.e. the test would see a missing bias correction or a wrong moment
    assert np.abs(gp["dec_ws"] - P["params"]["dec_ws"]).max() > 10 * lr
    G.ctx.tgnn_set_optimizer(0)            # back to SGD: a step with lr = 0 leaves the parameters alone
    before = G.params.numpy()
    G.step([batch_np(P, 50 * d.batch, 51 * d.batch)], lr=0.0, want=False)
    assert all(np.array_equal(before[n], x) for n, x in G.params.numpy().items())


@pytest.mark.parametrize("nrep", [1, 3])
def test_co_trained_static_memory_against_the_oracle(nrep):
    """tgnn_train_static (Sec. 3.1, static memory as a co-trained embedding table): the gradient of the static rows
    (dense [N, d_s], touched rows only) against the oracle on every checked step, and the table itself after 20 steps
    of sparse SGD on it together with SGD on the weights; with three memory replicas the rows of one node in different
    replicas add up."""
    import torch
    from gpu_common import rel_err
    P = custom_problem(n_nodes=120, E=3000, d_mem=32, d_time=16, d_edge=8, d_static=20, n_heads=2, k=6, batch=100, seed=3)
    d = P["d"]
    G = GpuSide(P, n_replicas=nrep); Or = OracleSide(P, n_replicas=nrep)
    gstat = torch.zeros(d.n_nodes, d.d_static, device="cuda")
    lr_s = 5.0     # (the rows' gradients are ~1e-5: a rate that moves the table by a few per cent over the test)
    G.ctx.tgnn_train_static(True, gstat, lr_s)
    Or.train_static(lr_s)
    n_steps = 20 // nrep + 2
    for s in range(n_steps):
        bl = [batch_np(P, (s * nrep + r) * d.batch, (s * nrep + r + 1) * d.batch) for r in range(nrep)]
        gstat.zero_()
        g = G.step(bl, lr=0.02)
        o = Or.step(bl, lr=0.02, gpu=g)
        compare_step(g, o, label=f"static nrep {nrep} step {s}")
        ref = o["g_static"]
        got = gstat.cpu().numpy()
        assert rel_err(got, ref) <= 1e-4, (s, rel_err(got, ref))
        assert np.all(got[np.all(ref == 0, axis=1)] == 0)              # untouched rows receive nothing
    assert rel_err(G.state.stat.cpu().numpy(), Or.static) <= 1e-4
    assert np.abs(Or.static - P["static"]).max() > 1e-3                # the table moved
    for r in range(nrep):
        compare_state(G.state_np(r), Or.states[r], label=f"replica {r}")
    G.ctx.tgnn_train_static(False)
    before = G.state.stat.clone()
    G.step([batch_np(P, 0, d.batch)], lr=0.0, want=False)
    assert torch.equal(before, G.state.stat)


@pytest.mark.parametrize("seed", list(range(40)))
def test_random_shapes_against_the_oracle(seed):
    """Seeded random widths, head counts, neighbour counts, batch sizes, negative-set counts and launch flags inside the
    library's limits (including k up to 32, one-column time encodings, no edge features, widths that are not multiples of
    anything): four consecutive steps each, every quantity of compare_step."""
    rng = np.random.default_rng(1000 + seed)
    H = int(rng.choice([1, 1, 2, 2, 3, 4, 5]))
    d_mem = H * int(rng.integers(1, max(2, 160 // H)))
    k = int(rng.choice([1, 2, 3, 5, 7, 10, 10, 12, 17, 32]))
    while 16 * (d_mem + k * (d_mem + 1) + 2 * H * k) > 64 * 1024:      # the library's limit on k * d_mem (tgnn_create)
        k -= 1
    shape = dict(n_nodes=int(rng.integers(12, 220)), E=0, d_mem=d_mem, d_time=int(rng.choice([1, 2, 5, 16, 33, 100, 140])),
                 d_edge=int(rng.choice([0, 1, 3, 16, 64, 172, 210])), d_static=int(rng.choice([0, 0, 1, 7, 20])),
                 n_heads=H, k=k, batch=int(rng.integers(3, 90)))
    shape["E"] = shape["batch"] * 5 + int(rng.integers(0, shape["batch"]))
    J = int(rng.choice([1, 1, 1, 2, 3]))
    flags = int(rng.choice([0, 0, 8, 16, 4]))
    P = custom_problem(**shape, seed=seed, ties=bool(rng.integers(0, 2)), self_loops=float(rng.choice([0.0, 0.1])),
                       neg_is_dst=float(rng.choice([0.0, 0.1])))
    d = P["d"]
    G = GpuSide(P, flags=flags, max_neg_sets=J); Or = OracleSide(P)
    for s in range(4):
        b = batch_np(P, s * d.batch, (s + 1) * d.batch)
        if J > 1:
            b["neg"] = rng.integers(0, d.n_nodes, (J, d.batch)).astype(np.int32)
        g = G.step([b], lr=0.03, n_neg_sets=J)
        o = Or.step([b], lr=0.03, gpu=g)
        compare_step(g, o, label=f"random shape {seed} {shape} J={J} flags={flags} step {s}")
    compare_state(G.state_np(), Or.states[0], label=f"random shape {seed}")
