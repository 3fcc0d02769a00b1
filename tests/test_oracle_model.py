"""Pins for the oracle's model pieces: closed forms of the time encoding, a library GRU cell and the
cell's limits, special cases of the attention layer, ln 2 for zero logits."""
import numpy as np
import pytest
import torch

import synth
from oracle import tgnn_oracle as O


def test_time_encoding_closed_forms():
    w = np.array([np.pi, 0.0, 2.0, 0.5]); b = np.array([0.0, 0.3, 0.0, -1.0])
    np.testing.assert_allclose(O.time_encode(0.0, w, b), np.cos(b), atol=0)
    out = O.time_encode(1.0, w, b)
    assert abs(out[0] + 1.0) < 1e-15 and out[1] == np.cos(0.3)
    # period 2 pi / w
    np.testing.assert_allclose(O.time_encode(np.array([1.3]), w[2:3], b[2:3]),
                               O.time_encode(np.array([1.3 + np.pi]), w[2:3], b[2:3]), atol=1e-14)
    # cos(0.5 * 2 - 1) = 1
    assert abs(O.time_encode(2.0, w, b)[3] - 1.0) < 1e-15
    # half period flips the sign (catches a dropped phase or a sin/cos mix-up)
    np.testing.assert_allclose(O.time_encode(np.array([0.7 + np.pi / 2.0]), w[2:3], b[2:3]),
                               -O.time_encode(np.array([0.7]), w[2:3], b[2:3]), atol=1e-14)
    assert O.time_encode(np.zeros((3, 2)), w, b).shape == (3, 2, 4)


def test_gru_matches_library_cell():
    rng = np.random.default_rng(0)
    d_in, d = 13, 5
    cell = torch.nn.GRUCell(d_in, d).double()
    x = rng.standard_normal((7, d_in)); h = rng.standard_normal((7, d))
    with torch.no_grad():
        ref = cell(torch.from_numpy(x), torch.from_numpy(h)).numpy()
    out = O.gru_cell(x, h, cell.weight_ih.detach().numpy(), cell.weight_hh.detach().numpy(),
                     cell.bias_ih.detach().numpy(), cell.bias_hh.detach().numpy())
    np.testing.assert_allclose(out, ref, rtol=1e-13, atol=1e-14)


def test_gru_limits():
    rng = np.random.default_rng(1)
    d_in, d = 6, 4
    wih = rng.standard_normal((3 * d, d_in)); whh = rng.standard_normal((3 * d, d))
    bih = rng.standard_normal(3 * d); bhh = rng.standard_normal(3 * d)
    x = rng.standard_normal((3, d_in)); h = rng.standard_normal((3, d))
    b2 = bhh.copy(); b2[d:2 * d] = 60.0                       # z -> 1: memory unchanged
    np.testing.assert_allclose(O.gru_cell(x, h, wih, whh, bih, b2), h, atol=1e-12)
    b3 = bhh.copy(); b3[:2 * d] = -60.0                       # r, z -> 0: h' = tanh(W_in x + b_in)
    ref = np.tanh(x @ wih[2 * d:].T + bih[2 * d:])
    np.testing.assert_allclose(O.gru_cell(x, h, wih, whh, bih, b3), ref, atol=1e-12)


def _attn_inputs(rng, R=6, k=4, d_m=8, d_s=0, d_e=3, d_t=4, H=2):
    d = synth.ModelDims(n_nodes=1, d_mem=d_m, d_time=d_t, d_edge=d_e, d_static=d_s, n_heads=H, k=k, batch=1)
    p = O.to_f64(synth.gen_params(d, seed=5, random_phase=True))
    x_root = rng.standard_normal((R, d.d_x)); x_nbr = rng.standard_normal((R, k, d.d_x))
    e_nbr = rng.standard_normal((R, k, d_e)); dt = rng.uniform(0, 50, (R, k))
    return d, p, x_root, x_nbr, e_nbr, dt


def _aggregated(p, cache):
    return cache["o"]


def test_attention_single_neighbour_returns_its_value():
    rng = np.random.default_rng(2)
    d, p, xr, xn, en, dt = _attn_inputs(rng)
    cnt = np.ones(xr.shape[0], np.int64)
    _, c = O.attention_fwd(p, xr, xn, en, dt, cnt, d.n_heads)
    np.testing.assert_allclose(c["o"], c["V"][:, 0, :], atol=1e-14)


def test_attention_uniform_when_keys_vanish_and_scale_is_sqrt_cnt():
    rng = np.random.default_rng(3)
    d, p, xr, xn, en, dt = _attn_inputs(rng)
    cnt = np.array([4, 3, 2, 1, 4, 0])
    p0 = dict(p); p0["wk"] = np.zeros_like(p["wk"])
    _, c = O.attention_fwd(p0, xr, xn, en, dt, cnt, d.n_heads)
    for r in range(6):
        ref = c["V"][r, :cnt[r]].mean(0) if cnt[r] else np.zeros(d.d_out)
        np.testing.assert_allclose(c["o"][r], ref, atol=1e-14)
    # probabilities sum to one; literal 1/sqrt(|N_v|) scale: recompute head 0 of root 0 by hand
    _, c = O.attention_fwd(p, xr, xn, en, dt, cnt, d.n_heads)
    np.testing.assert_allclose(c["pr"].sum(2)[cnt > 0], 1.0, atol=1e-14)
    dh = d.d_out // d.n_heads
    a = np.array([c["q"][0, :dh] @ c["K"][0, j, :dh] for j in range(4)]) / 2.0      # sqrt(4)
    pr = np.exp(a - a.max()); pr /= pr.sum()
    np.testing.assert_allclose(c["pr"][0, 0], pr, atol=1e-14)
    # root with no neighbour: aggregated vector is zero, the merge layer still sees x_v
    assert np.all(c["o"][5] == 0)
    z5 = np.maximum(p["wo"][:, d.d_out:] @ xr[5] + p["bo"], 0)
    np.testing.assert_allclose(O.attention_fwd(p, xr, xn, en, dt, cnt, d.n_heads)[0][5], z5, atol=1e-14)


def test_attention_permutation_invariance_and_padding_ignored():
    rng = np.random.default_rng(4)
    d, p, xr, xn, en, dt = _attn_inputs(rng)
    cnt = np.full(6, 3)
    z, _ = O.attention_fwd(p, xr, xn, en, dt, cnt, d.n_heads)
    perm = [2, 0, 1, 3]
    xn2, en2, dt2 = xn[:, perm].copy(), en[:, perm].copy(), dt[:, perm].copy()
    xn2[:, 3] = 99.0; en2[:, 3] = -7.0                         # garbage in the padded slot
    z2, _ = O.attention_fwd(p, xr, xn2, en2, dt2, cnt, d.n_heads)
    np.testing.assert_allclose(z, z2, atol=1e-13)


def test_attention_two_heads_equal_two_single_head_layers():
    rng = np.random.default_rng(5)
    d, p, xr, xn, en, dt = _attn_inputs(rng, H=2)
    cnt = np.array([4, 3, 2, 1, 4, 2])
    _, c2 = O.attention_fwd(p, xr, xn, en, dt, cnt, 2)
    dh = d.d_out // 2
    for hd in range(2):
        ph = dict(p)
        for n in ("wq", "wk", "wv"):
            ph[n] = p[n][hd * dh:(hd + 1) * dh]
        for n in ("bq", "bk", "bv"):
            ph[n] = p[n][hd * dh:(hd + 1) * dh]
        ph["wo"] = np.zeros((dh, dh + d.d_x)); ph["bo"] = np.zeros(dh)
        _, c1 = O.attention_fwd(ph, xr, xn, en, dt, cnt, 1)
        np.testing.assert_allclose(c1["o"], c2["o"][:, hd * dh:(hd + 1) * dh], atol=1e-14)


def test_attention_identical_keys_and_query_phase():
    rng = np.random.default_rng(6)
    d, p, xr, xn, en, dt = _attn_inputs(rng)
    xn[:] = xn[:, :1]; en[:] = en[:, :1]; dt[:] = dt[:, :1]
    cnt = np.full(6, 4)
    _, c = O.attention_fwd(p, xr, xn, en, dt, cnt, d.n_heads)
    np.testing.assert_allclose(c["o"], c["V"][:, 0], atol=1e-13)
    # the query sees Phi(0) = cos(b)
    np.testing.assert_allclose(c["q_in"][:, d.d_x:], np.broadcast_to(np.cos(p["time_b"]), (6, d.d_time)))
    # key layout {x_w || e_vw || Phi(dt)}
    np.testing.assert_allclose(c["c_in"][2, 1, d.d_x:d.d_x + d.d_edge], en[2, 1])
    np.testing.assert_allclose(c["c_in"][2, 1, d.d_x + d.d_edge:], np.cos(dt[2, 1] * p["time_w"] + p["time_b"]))


def test_decoder_zero_logits_give_ln2_and_softplus_is_stable():
    d = synth.ModelDims(n_nodes=1, d_mem=6, d_time=2, d_edge=0, d_static=0, n_heads=1, k=1, batch=1)
    p = O.to_f64(synth.gen_params(d, seed=1))
    p["dec_w2"][:] = 0; p["dec_b2"][:] = 0
    rng = np.random.default_rng(0)
    z = rng.standard_normal((3, 5, 6))
    loss, logits, _ = O.decoder_loss(p, z[0], z[1], z[2])
    assert np.all(logits == 0) and abs(loss - np.log(2)) < 1e-15
    p["dec_b2"][:] = 50.0
    loss, logits, _ = O.decoder_loss(p, z[0], z[1], z[2])
    assert np.isfinite(loss) and abs(loss - 0.5 * (np.log1p(np.exp(-50)) + 50 + np.log1p(np.exp(-50)))) < 1e-12
    p["dec_b2"][:] = -50.0
    loss, _, _ = O.decoder_loss(p, z[0], z[1], z[2])
    assert abs(loss - 0.5 * (50 + 2 * np.log1p(np.exp(-50)))) < 1e-12
