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
    adj = O.build_adjacency(src, dst, ts, n)
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
