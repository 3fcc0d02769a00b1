"""Pins of the oracle's edge-classification head and of its reciprocal rank (Sec. 4 "Datasets": the 56-class
multi-label task, and the mean reciprocal rank of the true destination among 49 sampled ones)."""
import math

import numpy as np

from oracle import tgnn_oracle as O
from test_oracle_step import tiny_problem, warm_state, batch_of
import synth


def _head(d, C, rng):
    return dict(dec_ws=rng.standard_normal((d, d)), dec_wd=rng.standard_normal((d, d)), dec_b1=rng.standard_normal(d),
                dec_w2=rng.standard_normal((C, d)), dec_b2=rng.standard_normal(C))


def test_zero_output_layer_gives_ln2_whatever_the_labels():
    rng = np.random.default_rng(0)
    p = _head(5, 7, rng); p["dec_w2"][:] = 0; p["dec_b2"][:] = 0
    y = (rng.random((9, 7)) < 0.3).astype(float)
    loss, logits, _ = O.edge_class_loss(p, rng.standard_normal((9, 5)), rng.standard_normal((9, 5)), y)
    assert logits.shape == (9, 7) and not logits.any()
    assert abs(loss - math.log(2.0)) < 1e-15


def test_one_event_by_hand():
    # z_src = (1, 0), z_dst = (0, 2), W_s = I, W_d = I, b1 = (0, -3): hidden = ReLU((1, 2) + (0, -3)) = (1, 0)
    p = dict(dec_ws=np.eye(2), dec_wd=np.eye(2), dec_b1=np.array([0.0, -3.0]),
             dec_w2=np.array([[2.0, 5.0], [-1.0, 5.0], [0.0, 5.0]]), dec_b2=np.array([0.5, 0.0, -0.25]))
    y = np.array([[1.0, 0.0, 1.0]])
    loss, logits, cache = O.edge_class_loss(p, np.array([[1.0, 0.0]]), np.array([[0.0, 2.0]]), y)
    assert np.allclose(logits, [[2.5, -1.0, -0.25]], atol=1e-15)         # W2[c, 0] * 1 + b2[c]
    bce = [math.log1p(math.exp(-2.5)), math.log1p(math.exp(-1.0)), math.log1p(math.exp(0.25))]   # y=1, y=0, y=1
    assert abs(loss - sum(bce) / 3) < 1e-15
    g, dzs, dzd = O.edge_class_bwd(p, cache, logits)
    sig = lambda x: 1.0 / (1.0 + math.exp(-x))
    dl = np.array([sig(2.5) - 1, sig(-1.0), sig(-0.25) - 1]) / 3
    assert np.allclose(g["dec_b2"], dl, atol=1e-15)
    assert np.allclose(g["dec_w2"], np.outer(dl, [1.0, 0.0]), atol=1e-15)
    dh = np.array([dl @ p["dec_w2"][:, 0], 0.0])                          # the second hidden unit is gated off
    assert np.allclose(g["dec_b1"], dh, atol=1e-15) and np.allclose(dzs, [dh], atol=1e-15) and np.allclose(dzd, [dh], atol=1e-15)
    assert np.allclose(g["dec_ws"], np.outer(dh, [1.0, 0.0]), atol=1e-15)
    assert np.allclose(g["dec_wd"], np.outer(dh, [0.0, 2.0]), atol=1e-15)


def test_one_class_with_true_label_is_the_link_loss_of_the_true_pairs():
    rng = np.random.default_rng(1)
    p = _head(4, 1, rng)
    zs, zd, zn = (rng.standard_normal((6, 4)) for _ in range(3))
    loss, logits, _ = O.edge_class_loss(p, zs, zd, np.ones((6, 1)))
    q = dict(p, dec_w2=p["dec_w2"][0], dec_b2=p["dec_b2"])
    _, link_logits, _ = O.decoder_loss(q, zs, zd, zn)
    assert np.allclose(logits[:, 0], link_logits[:6], atol=1e-14)
    assert abs(loss - np.log1p(np.exp(-link_logits[:6])).mean()) < 1e-14


def test_edge_classification_step_by_finite_differences():
    P = tiny_problem(seed=21, n=90)
    d = P["d"]
    C = 5
    rng = np.random.default_rng(2)
    p = dict(P["p"]); p["dec_w2"] = rng.uniform(-0.5, 0.5, (C, d.d_mem)); p["dec_b2"] = rng.uniform(-0.5, 0.5, C)
    st = warm_state(P, 10)
    labels = synth.gen_labels(len(P["src"]), C, 2, seed=3).astype(np.float64)
    bt = batch_of(P, 10 * d.batch, 11 * d.batch); bt["labels"] = labels[10 * d.batch:11 * d.batch]
    assert np.all(bt["labels"].sum(1) == 2)
    fb = O.forward_backward(st, P["adj"], P["efeat"], P["static"], p, bt, d.k, d.n_heads)
    assert fb["logits"].shape == (d.batch, C) and len(fb["cnt"]) == 2 * d.batch

    def loss_with(name, idx, val):
        q = dict(p); a = q[name].copy(); a[idx] = val; q[name] = a
        return O.forward_backward(st, P["adj"], P["efeat"], P["static"], q, bt, d.k, d.n_heads, want_grads=False)["loss"]

    for name in O.PARAM_NAMES:
        g = fb["grads"][name]
        assert g.shape == p[name].shape and np.abs(g).max() > 0, name
        for i in rng.choice(g.size, min(g.size, 10), replace=False):
            idx = np.unravel_index(i, g.shape); x0 = p[name][idx]; h = 1e-6
            fd = (loss_with(name, idx, x0 + h) - loss_with(name, idx, x0 - h)) / (2 * h)
            assert abs(fd - g[idx]) <= 2e-7 * max(1.0, abs(fd)) + 1e-9, (name, idx, fd, g[idx])
    # the write-back of a classification batch is that of its events: same winners as the link-prediction batch
    a = copy_state(st); b = copy_state(st)
    w1 = O.apply_writeback(a, bt, fb)
    bl = batch_of(P, 10 * d.batch, 11 * d.batch)
    w2 = O.apply_writeback(b, bl, O.forward_backward(st, P["adj"], P["efeat"], P["static"], P["p"], bl, d.k, d.n_heads))
    assert np.array_equal(w1, w2) and all(np.array_equal(a[k], b[k]) for k in a)


def copy_state(st):
    return {k: v.copy() for k, v in st.items()}


def test_reciprocal_rank_by_hand():
    # event 0: two negatives above the true score -> rank 3; event 1: none above, one tie -> 1.5; event 2: all below -> 1
    st = np.array([0.2, 1.0, 5.0])
    sn = np.array([[0.3, 1.0, 4.0], [0.9, -2.0, 4.9], [0.1, 0.5, -7.0]])
    rank, mrr = O.reciprocal_rank(st, sn)
    assert rank.tolist() == [3.0, 1.5, 1.0]
    assert abs(mrr - (1 / 3 + 1 / 1.5 + 1.0) / 3) < 1e-15
    # 49 negatives, true score in the middle: rank = 1 + the count above
    rng = np.random.default_rng(0)
    sn = rng.standard_normal((49, 1)); s0 = np.array([0.0])
    rank, _ = O.reciprocal_rank(s0, sn)
    assert rank[0] == 1 + sorted(sn[:, 0].tolist() + [0.0], reverse=True).index(0.0)


def test_labels_generator_shape():
    y = synth.gen_labels(1000, 56, 6, seed=1)
    assert y.shape == (1000, 56) and y.dtype == np.float32 and np.all(y.sum(1) == 6) and set(np.unique(y)) == {0.0, 1.0}
    assert y[:, 0].mean() > 3 * y[:, 55].mean()          # skewed class popularity


def test_f1_micro_counts_by_hand():
    logits = np.array([[2.0, -1.0, 0.5, -3.0], [0.0, 1.0, -0.1, 4.0]])
    labels = np.array([[1, 0, 0, 1], [1, 1, 0, 0]], dtype=float)
    # predicted: (0,0) (0,2) (1,1) (1,3);  true: (0,0) (0,3) (1,0) (1,1);  a logit of exactly 0 is not a prediction
    tp, fp, fn = O.f1_micro_counts(logits, labels)
    assert (tp, fp, fn) == (2, 2, 2)
    assert abs(2 * tp / (2 * tp + fp + fn) - 0.5) < 1e-15
    assert O.f1_micro_counts(np.full((3, 5), 7.0), np.ones((3, 5))) == (15, 0, 0)
    assert O.f1_micro_counts(np.full((3, 5), -7.0), np.ones((3, 5))) == (0, 0, 15)
