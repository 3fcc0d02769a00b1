"""Pins for the oracle's training step: central finite differences for every parameter tensor,
brute-force last-writer-wins write-back, and the invariants the paper states (zero-initialised
memory, supporting nodes never written, gradients stop at the stored memory)."""
import copy

import numpy as np
import pytest

import synth
from oracle import tgnn_oracle as O


def tiny_problem(seed=0, n=40, E=400, d_m=6, d_t=4, d_e=3, d_s=2, H=2, k=3, B=12, tmax=30.0):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, E); dst = (src + rng.integers(1, n, E)) % n
    ts = np.sort(rng.uniform(0, tmax, E))
    efeat = rng.standard_normal((E, d_e)).astype(np.float32)
    static = (0.1 * rng.standard_normal((n, d_s))).astype(np.float32) if d_s else None
    d = synth.ModelDims(n_nodes=n, d_mem=d_m, d_time=d_t, d_edge=d_e, d_static=d_s, n_heads=H, k=k, batch=B)
    p = O.to_f64(synth.gen_params(d, seed=seed, random_phase=True))
    p["time_w"] = rng.uniform(0.05, 1.0, d_t)
    neg = rng.integers(0, n, E)
    adj = O.event_list(src, dst, ts)          # neighbours by the plain scan of the event list
    return dict(src=src, dst=dst, ts=ts, efeat=efeat, static=static, d=d, p=p, neg=neg, adj=adj)


def batch_of(P, lo, hi):
    return dict(src=P["src"][lo:hi], dst=P["dst"][lo:hi], neg=P["neg"][lo:hi], eid=np.arange(lo, hi),
                t=P["ts"][lo:hi])


def warm_state(P, n_batches):
    d = P["d"]
    st = O.new_state(d.n_nodes, d.d_mem)
    for b in range(n_batches):
        O.train_step([st], P["adj"], P["efeat"], P["static"], P["p"], [batch_of(P, b * d.batch, (b + 1) * d.batch)],
                     d.k, d.n_heads)
    return st


@pytest.mark.parametrize("dt_source,d_s,H", [(0, 2, 2), (1, 0, 1), (0, 0, 3)])
def test_finite_difference_gradients(dt_source, d_s, H):
    P = tiny_problem(seed=3 + dt_source, n=110, d_s=d_s, H=H)
    d = P["d"]
    st = warm_state(P, 12)
    assert (st["mail_eid"] >= 0).sum() > 20
    bt = batch_of(P, 12 * d.batch, 13 * d.batch)
    fb = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], bt, d.k, d.n_heads, dt_source)
    assert fb["cnt"].max() == d.k and fb["cnt"].min() < d.k

    def loss_with(name, idx, val):
        q = dict(P["p"]); a = q[name].copy(); a[idx] = val; q[name] = a
        return O.forward_backward(st, P["adj"], P["efeat"], P["static"], q, bt, d.k, d.n_heads, dt_source,
                                  want_grads=False)["loss"]

    rng = np.random.default_rng(0)
    for name in O.PARAM_NAMES:
        g = fb["grads"][name]
        assert g.shape == P["p"][name].shape
        flat = [np.unravel_index(i, g.shape) for i in rng.choice(g.size, min(g.size, 12), replace=False)]
        assert np.abs(g).max() > 0, name
        for idx in flat:
            x0 = P["p"][name][idx]; h = 1e-6
            fd = (loss_with(name, idx, x0 + h) - loss_with(name, idx, x0 - h)) / (2 * h)
            assert abs(fd - g[idx]) <= 2e-7 * max(1.0, abs(fd)) + 1e-9, (name, idx, fd, g[idx])


def test_loss_scale_and_replica_sum():
    P = tiny_problem(seed=9)
    d = P["d"]
    st = warm_state(P, 6)
    st2 = copy.deepcopy(st)
    b1 = batch_of(P, 72, 84); b2 = batch_of(P, 84, 96)
    o1 = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], b1, d.k, d.n_heads)
    o2 = O.forward_backward(st2, P["adj"], P["efeat"], P["static"], P["p"], b2, d.k, d.n_heads)
    res = O.train_step([st, st2], P["adj"], P["efeat"], P["static"], P["p"], [b1, b2], d.k, d.n_heads)
    assert abs(res["loss"] - 0.5 * (o1["loss"] + o2["loss"])) < 1e-15
    for n in O.PARAM_NAMES:
        np.testing.assert_allclose(res["grads"][n], o1["grads"][n] + o2["grads"][n], rtol=1e-13, atol=1e-16)


def test_writeback_last_event_wins_and_only_roots_change():
    P = tiny_problem(seed=5, n=15, B=40)             # few nodes: many repeats inside a batch
    d = P["d"]
    st = warm_state(P, 3)
    before = copy.deepcopy(st)
    bt = batch_of(P, 120, 160)
    fb = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], bt, d.k, d.n_heads)
    win = O.apply_writeback(st, bt, fb)
    B = 40
    touched = set(bt["src"].tolist()) | set(bt["dst"].tolist())
    assert win.sum() == len(touched)
    for node in range(d.n_nodes):
        occ = [(i, 0) for i in range(B) if bt["src"][i] == node] + [(i, 1) for i in range(B) if bt["dst"][i] == node]
        if not occ:
            for key in st:
                assert np.array_equal(st[key][node], before[key][node])
            continue
        i, role = max(occ)
        assert win[role * B + i] == 1
        me, other = (i, B + i) if role == 0 else (B + i, i)
        assert np.array_equal(st["mem"][node], fb["s_new"][me])
        assert np.array_equal(st["mail"][node], np.concatenate([fb["s_new"][me], fb["s_new"][other]]))
        assert st["mail_eid"][node] == bt["eid"][i] and st["mail_ts"][node] == bt["t"][i]
        assert st["mem_ts"][node] == fb["tau"][me]
        # every occurrence of a node carries the same s' (computed from the same stored state)
        for (i2, r2) in occ:
            assert np.array_equal(fb["s_new"][r2 * B + i2], fb["s_new"][me])
    # a negative destination that is no positive endpoint is untouched
    only_neg = set(bt["neg"].tolist()) - touched
    for node in only_neg:
        assert np.array_equal(st["mem"][node], before["mem"][node])


def test_first_batch_reads_zeros_and_time_differences_nonnegative():
    P = tiny_problem(seed=6)
    d = P["d"]
    st = O.new_state(d.n_nodes, d.d_mem)
    fb = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], batch_of(P, 0, d.batch), d.k, d.n_heads)
    assert np.all(fb["s_new"] == 0) and np.all(fb["tau"] == 0)
    for name in ("gru_wih", "gru_whh", "gru_bih", "gru_bhh"):
        assert np.all(fb["grads"][name] == 0)          # no mail consumed -> no GRU cell evaluated
    st = warm_state(P, 10)
    for src_mode in (0, 1):
        fb = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], batch_of(P, 120, 132), d.k,
                                d.n_heads, src_mode)
        assert np.all(fb["dt_nbr"] >= 0)
    assert np.all(st["mail_ts"] >= st["mem_ts"])


def test_stored_state_is_a_constant_of_the_step_and_split_run_is_deterministic():
    P = tiny_problem(seed=7)
    d = P["d"]
    full = warm_state(P, 10)
    half = warm_state(P, 5)
    snap = copy.deepcopy(half)
    for b in range(5, 10):
        O.train_step([snap], P["adj"], P["efeat"], P["static"], P["p"], [batch_of(P, b * d.batch, (b + 1) * d.batch)],
                     d.k, d.n_heads)
    for key in full:
        assert np.array_equal(full[key], snap[key])
    st = copy.deepcopy(full)
    O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], batch_of(P, 120, 132), d.k, d.n_heads)
    for key in full:
        assert np.array_equal(full[key], st[key])      # forward/backward never writes the state


def test_sgd_freezes_time_encoding():
    P = tiny_problem(seed=8)
    d = P["d"]
    st = warm_state(P, 6)
    p0 = copy.deepcopy(P["p"])
    res = O.train_step([st], P["adj"], P["efeat"], P["static"], P["p"], [batch_of(P, 72, 84)], d.k, d.n_heads, lr=0.1)
    assert np.array_equal(P["p"]["time_w"], p0["time_w"]) and np.array_equal(P["p"]["time_b"], p0["time_b"])
    np.testing.assert_allclose(P["p"]["wk"], p0["wk"] - 0.1 * res["grads"]["wk"], rtol=0, atol=1e-15)


def _hand_built_step(dt_source=0, mail_ts0=5.0):
    """Four nodes, two events, a state written out by hand so that every time difference of the step is known:
         event 0: 1 -> 2 at t = 2          event 1: 0 -> 1 at t = 7 (the batch; negative destination: node 3)
         node 0: memory updated at 4, mail of time mail_ts0 (default 5)   -> mail difference 1
         node 1: memory updated at 1, mail of time 6                      -> mail difference 5
         node 2: memory updated at 2.5, mail of time 6                    -> used memory is as of 6
       Root 1 (node 1 at t = 7) has one earlier event, event 0, with neighbour 2: key difference 7 - 6 = 1
       (memory-time reading) or 7 - 2 = 5 (edge-time reading).  Roots 0 and 3 have no earlier event."""
    d = synth.ModelDims(n_nodes=4, d_mem=2, d_time=3, d_edge=1, d_static=0, n_heads=1, k=2, batch=1)
    p = O.to_f64(synth.gen_params(d, seed=11))
    p["time_w"] = np.array([np.pi / 2, np.pi, 0.25]); p["time_b"] = np.array([np.pi / 2, 0.0, 1.0])
    rng = np.random.default_rng(0)
    st = O.new_state(4, 2)
    st["mem"][:] = rng.standard_normal((4, 2)); st["mail"][:] = rng.standard_normal((4, 4))
    st["mem_ts"][:] = [4.0, 1.0, 2.5, 0.0]; st["mail_ts"][:] = [mail_ts0, 6.0, 6.0, 0.0]
    st["mail_eid"][:] = [0, 0, 0, -1]
    g = O.event_list([1, 0], [2, 1], [2.0, 7.0])
    efeat = np.array([[0.5], [-0.25]], np.float32)
    bt = dict(src=np.array([0]), dst=np.array([1]), neg=np.array([3]), eid=np.array([1]), t=np.array([7.0]))
    return O.forward_backward(st, g, efeat, None, p, bt, d.k, d.n_heads, dt_source), d


def test_time_encoding_inside_the_step_hand_values():
    """Eq. 1-2 and 5-6 as the step evaluates them, against values worked out by hand with non-zero phases and
    time differences whose sign matters: w = (pi/2, pi, 1/4), b = (pi/2, 0, 1)."""
    fb, d = _hand_built_step()
    assert fb["nbr"].tolist() == [[-1, -1], [2, -1], [-1, -1]]
    phi_gru = fb["gru_x"][:, 2 * d.d_mem:2 * d.d_mem + d.d_time]
    # slot 0 = root node 0: mail time - memory time = 1: cos(pi/2 + pi/2) = -1, cos(pi) = -1, cos(1.25)
    np.testing.assert_allclose(phi_gru[0], [-1.0, -1.0, 0.3153223623952687], atol=1e-15)
    # slot 1 = root node 1: difference 5: cos(3 pi) = -1, cos(5 pi) = -1, cos(2.25)
    np.testing.assert_allclose(phi_gru[1], [-1.0, -1.0, -0.6281736227227391], atol=1e-14)
    # slot 2 = negative root node 3, no mail: difference taken as 0 (and the cell is not applied)
    np.testing.assert_allclose(phi_gru[2], [0.0, 1.0, 0.5403023058681398], atol=1e-15)
    # key of root 1's neighbour: query time 7 - time of the neighbour's memory as used (its mail time 6) = 1
    phi_key = fb["c_in"][1, 0, d.d_x + d.d_edge:]
    np.testing.assert_allclose(phi_key, [-1.0, -1.0, 0.3153223623952687], atol=1e-15)
    assert fb["c_in"][1, 0, d.d_x] == 0.5                                  # its edge feature: event 0
    # the query encodes a time difference of zero: cos(b) = (0, 1, cos 1)
    np.testing.assert_allclose(fb["q_in"][:, d.d_x:], np.tile([0.0, 1.0, 0.5403023058681398], (3, 1)), atol=1e-15)
    # edge-time reading: 7 - 2 = 5
    fb1, _ = _hand_built_step(dt_source=1)
    np.testing.assert_allclose(fb1["c_in"][1, 0, d.d_x + d.d_edge:], [-1.0, -1.0, -0.6281736227227391], atol=1e-14)
    # the mail's edge feature sits after the time encoding in the GRU input (Eq. 1-2 order)
    assert fb["gru_x"][0, -1] == 0.5


def test_half_period_flips_the_sign_through_the_step():
    fb_a, d = _hand_built_step(mail_ts0=5.0)      # difference 1
    fb_b, _ = _hand_built_step(mail_ts0=6.0)      # difference 2: half a period of w = pi, a quarter of w = pi/2
    c = 2 * d.d_mem
    assert abs(fb_a["gru_x"][0, c + 1] + fb_b["gru_x"][0, c + 1]) < 1e-15 and abs(fb_a["gru_x"][0, c + 1] + 1.0) < 1e-15
    np.testing.assert_allclose(fb_b["gru_x"][0, c], np.cos(np.pi + np.pi / 2), atol=1e-15)   # ~ 0: a quarter period on
    assert np.abs(fb_a["s_new"][0] - fb_b["s_new"][0]).max() > 1e-3     # and the updated memory of node 0 follows


def test_time_encoding_derivative_by_finite_differences():
    w = np.array([0.3, 2.0, 0.0]); b = np.array([0.4, -1.0, 0.7])
    for delta in (0.0, 1.7, 13.0):
        h = 1e-6
        fd_b = (O.time_encode(delta, w, b + h) - O.time_encode(delta, w, b - h)) / (2 * h)
        np.testing.assert_allclose(O.time_encode_darg(delta, w, b), fd_b, atol=1e-9)
        fd_w = (O.time_encode(delta, w + h, b) - O.time_encode(delta, w - h, b)) / (2 * h)
        np.testing.assert_allclose(O.time_encode_darg(delta, w, b) * delta, fd_w, atol=1e-8)


def test_epoch_parallel_step_is_the_sum_of_its_trainers():
    """Sec. 3.2.2: J trainers share one positive mini-batch and differ in their negative destinations.  One step with
    J negative sets must give the mean of the J single-set losses and the sum of their gradients (each computed by the
    plain step from the same state), the same sampled neighbours for the shared roots, and -- since only the positive
    endpoints are written -- the same memory and mails."""
    P = tiny_problem(seed=12, n=60)
    d = P["d"]
    st = warm_state(P, 8)
    lo, hi = 8 * d.batch, 9 * d.batch
    rng = np.random.default_rng(1)
    J = 3
    negs = rng.integers(0, d.n_nodes, (J, d.batch))
    bt = batch_of(P, lo, hi)
    singles = []
    for g in range(J):
        b1 = dict(bt, neg=negs[g])
        singles.append(O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], b1, d.k, d.n_heads))
    multi = O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], dict(bt, neg=negs), d.k, d.n_heads)
    B = d.batch
    assert multi["logits"].shape == ((1 + J) * B,) and multi["cnt"].shape == ((2 + J) * B,)
    assert abs(multi["loss"] - np.mean([s_["loss"] for s_ in singles])) < 1e-14
    for name in O.PARAM_NAMES:
        np.testing.assert_allclose(multi["grads"][name], sum(s_["grads"][name] for s_ in singles), rtol=1e-11, atol=1e-15)
    for g in range(J):
        np.testing.assert_allclose(multi["logits"][:B], singles[g]["logits"][:B], atol=1e-14)
        np.testing.assert_allclose(multi["logits"][(1 + g) * B:(2 + g) * B], singles[g]["logits"][B:], atol=1e-14)
        assert np.array_equal(multi["nbr"][(2 + g) * B:(3 + g) * B], singles[g]["nbr"][2 * B:])
    st_a = copy.deepcopy(st); st_b = copy.deepcopy(st)
    O.apply_writeback(st_a, dict(bt, neg=negs), multi)
    O.apply_writeback(st_b, dict(bt, neg=negs[0]), singles[0])
    for key in st_a:
        assert np.array_equal(st_a[key], st_b[key])


def test_static_memory_gradient_by_finite_differences():
    """Co-trained static memory (Sec. 3.1): d loss / d static[w, c] against central differences, for nodes that are
    roots, supporting nodes, both (several slots), and nodes the batch does not touch (zero)."""
    P = tiny_problem(seed=21, n=50, d_s=3)
    d = P["d"]
    st = warm_state(P, 10)
    bt = batch_of(P, 10 * d.batch, 11 * d.batch)
    static = P["static"].astype(np.float64)
    fb = O.forward_backward(st, P["adj"], P["efeat"], static, P["p"], bt, d.k, d.n_heads)
    g = fb["g_static"]
    assert g.shape == static.shape
    refs = np.bincount(np.concatenate([np.concatenate([bt["src"], bt["dst"], bt["neg"]]), fb["nbr"][fb["nbr"] >= 0]]),
                       minlength=d.n_nodes)
    assert refs.max() >= 3 and (refs == 0).any()
    assert np.all(g[refs == 0] == 0) and np.abs(g[refs > 0]).max() > 0
    rng = np.random.default_rng(0)
    nodes = list(rng.choice(np.nonzero(refs > 0)[0], 8, replace=False)) + [int(np.argmax(refs))]
    for w in nodes:
        for c in range(static.shape[1]):
            h = 1e-6
            sp = static.copy(); sp[w, c] += h
            sm = static.copy(); sm[w, c] -= h
            lp = O.forward_backward(st, P["adj"], P["efeat"], sp, P["p"], bt, d.k, d.n_heads, want_grads=False)["loss"]
            lm = O.forward_backward(st, P["adj"], P["efeat"], sm, P["p"], bt, d.k, d.n_heads, want_grads=False)["loss"]
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[w, c]) <= 2e-7 * max(1.0, abs(fd)) + 1e-9, (w, c, fd, g[w, c])


def test_adam_two_steps_by_hand():
    """Two Adam steps on one scalar, worked out by hand with beta1 = 0.5, beta2 = 0.75, eps = 0, lr = 0.1, gradients
    g1 = 2, g2 = -1:
      step 1: m = 1, v = 1;       m^ = 1 / (1 - 0.5) = 2,      v^ = 1 / (1 - 0.75) = 4,        p = 1 - 0.1 * 2 / 2 = 0.9
      step 2: m = 0, v = 1;       m^ = 0                                                         p stays 0.9
    and a third with g3 = 4: m = 2, v = 4.75; m^ = 2 / (1 - 1/8) = 16/7, v^ = 4.75 / (1 - 27/64) = 304/37,
      p = 0.9 - 0.1 * (16/7) / sqrt(304/37)."""
    p = {n: np.array([1.0]) for n in O.PARAM_NAMES}
    st = O.adam_init(p)
    for g, want in ((2.0, 0.9), (-1.0, 0.9), (4.0, 0.9 - 0.1 * (16 / 7) / np.sqrt(304 / 37))):
        O.adam(p, {n: np.array([g]) for n in O.PARAM_NAMES}, st, 0.1, 0.5, 0.75, 0.0)
        assert abs(p["wq"][0] - want) < 1e-15 and abs(p["dec_b2"][0] - want) < 1e-15
        assert p["time_w"][0] == 1.0 and p["time_b"][0] == 1.0          # frozen
    assert st["t"] == 3
    # with eps: p -= lr m^ / (sqrt(v^) + eps)
    p = {n: np.array([0.0]) for n in O.PARAM_NAMES}
    st = O.adam_init(p)
    O.adam(p, {n: np.array([3.0]) for n in O.PARAM_NAMES}, st, 1.0, 0.9, 0.999, 1.0)
    assert abs(p["wk"][0] + 3.0 / (3.0 + 1.0)) < 1e-15
