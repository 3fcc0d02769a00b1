"""GPU parity of the individual C-ABI entry points against the CPU oracle (and brute force) on seeded
inputs: sampler and write-back winners bit-exact, gathers bit-exact, floating point within 1e-4."""
import numpy as np
import pytest
import torch

import synth
from gpu_common import FP32_EPS, TOL, OracleSide, batch_np, custom_problem, make_problem, rel_err
from oracle import tgnn_oracle as O

pytestmark = pytest.mark.gpu


def dev(a, dt=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.to("cuda", dtype=dt) if dt else t.to("cuda")


def make_ctx(P, n_replicas=1, dt_source=0, max_batch=None):
    from paper_2307_07649_amd import tgnn
    d = P["d"]
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, max_batch or d.batch,
                       n_replicas=n_replicas, dt_source=dt_source)
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
    return tgnn, ctx, graph


def brute_force(src, dst, ts, node, t, k):
    m = ((src == node) | (dst == node)) & (ts < t)
    idx = np.nonzero(m)[0]
    out = []
    for e in idx:                       # a self loop is listed twice
        if src[e] == node:
            out.append((ts[e], e, dst[e]))
        if dst[e] == node:
            out.append((ts[e], e, src[e]))
    out.sort(key=lambda c: (c[0], c[1]))
    return out[::-1][:k]


@pytest.mark.parametrize("case", ["C0", "ties", "C1"])
def test_sample_recent(case):
    if case == "ties":
        P = custom_problem(n_nodes=40, E=3000, d_mem=8, d_time=4, d_edge=2, d_static=0, n_heads=1, k=7, batch=64,
                           tmax=50, ties=True)
    else:
        P = make_problem(case)
    tgnn, ctx, graph = make_ctx(P, max_batch=4096)
    d = P["d"]
    rng = np.random.default_rng(1)
    n = 5000
    qn = rng.integers(0, d.n_nodes, n).astype(np.int32)
    qt = rng.uniform(-1.0, P["ts"][-1] * 1.05, n)
    if case == "ties":
        qt = np.round(qt)
    ev = rng.integers(0, P["E"], n // 2)                         # half the queries sit exactly on event times
    qn[:n // 2] = P["src"][ev]; qt[:n // 2] = P["ts"][ev]
    nbr, eid, ts, cnt = ctx.tgnn_sample_recent(graph, dev(qn), dev(qt))
    o_nbr, o_eid, o_ts, o_cnt = O.sample_recent(P["src"], P["dst"], P["ts"], qn, qt, d.k)     # the scan of the event list
    assert np.array_equal(cnt.cpu().numpy(), o_cnt)
    assert np.array_equal(nbr.cpu().numpy(), o_nbr) and np.array_equal(eid.cpu().numpy(), o_eid)
    assert np.array_equal(ts.cpu().numpy(), o_ts)
    m = np.arange(d.k)[None] < o_cnt[:, None]
    assert np.all(ts.cpu().numpy()[m] < np.broadcast_to(qt[:, None], m.shape)[m])        # strictly in the past
    for r in rng.integers(0, n, 40):                             # independent brute force on the raw event list
        ref = brute_force(P["src"], P["dst"], P["ts"], qn[r], qt[r], d.k)
        got = list(zip(ts[r].tolist(), eid[r].tolist(), nbr[r].tolist()))[:len(ref)]
        assert cnt[r].item() == len(ref) and got == [(a, int(b), int(c)) for a, b, c in ref]


def test_sample_recent_empty_and_degenerate():
    P = custom_problem(n_nodes=20, E=50, d_mem=8, d_time=4, d_edge=2, d_static=0, n_heads=1, k=10, batch=8)
    P["src"][:] = np.minimum(P["src"], 9); P["dst"][:] = np.minimum(P["dst"], 9)     # nodes 10..19 isolated
    tgnn, ctx, graph = make_ctx(P)
    qn = dev(np.array([15, 3, 3, 0], np.int32)); qt = dev(np.array([50.0, -5.0, 1e9, P["ts"][0]]))
    nbr, eid, ts, cnt = ctx.tgnn_sample_recent(graph, qn, qt)
    c = cnt.cpu().numpy()
    assert c[0] == 0 and c[1] == 0 and np.all(nbr[:2].cpu().numpy() == -1) and np.all(ts[:2].cpu().numpy() == 0)
    deg3 = int(((P["src"] == 3).astype(int) + (P["dst"] == 3).astype(int)).sum())
    assert c[2] == min(10, deg3)
    e = ctx.tgnn_sample_recent(graph, qn[:0], qt[:0])            # zero queries is a no-op
    assert e[0].shape[0] == 0


def warm(P, n_batches, n_replicas=1):
    Or = OracleSide(P, n_replicas)
    for s in range(n_batches):
        Or.step([batch_np(P, s * P["d"].batch, (s + 1) * P["d"].batch)])
    return Or


def state_to_gpu(tgnn, P, ostate, n_replicas=1, replica=0):
    d = P["d"]
    st = tgnn.State(d.n_nodes, d.d_mem, n_replicas, P["static"])
    s = slice(replica * d.n_nodes, (replica + 1) * d.n_nodes)
    st.mem[s] = dev(ostate["mem"], torch.float32); st.mail[s] = dev(ostate["mail"], torch.float32)
    st.mem_ts[s] = dev(ostate["mem_ts"]); st.mail_ts[s] = dev(ostate["mail_ts"])
    st.mail_eid[s] = dev(ostate["mail_eid"], torch.int32)
    return st


@pytest.mark.parametrize("shape", [
    dict(n_nodes=1500, E=3000, d_mem=100, d_time=100, d_edge=172, d_static=0, n_heads=2, k=10, batch=200),
    dict(n_nodes=700, E=1500, d_mem=32, d_time=20, d_edge=186, d_static=0, n_heads=2, k=5, batch=100),
    dict(n_nodes=500, E=900, d_mem=6, d_time=3, d_edge=5, d_static=0, n_heads=1, k=4, batch=60),
])
def test_gather_then_gru_update(shape):
    P = custom_problem(**shape)
    d = P["d"]
    Or = warm(P, 8)
    tgnn, ctx, graph = make_ctx(P, n_replicas=2)
    st = state_to_gpu(tgnn, P, Or.states[0], n_replicas=2, replica=1)
    rng = np.random.default_rng(0)
    slots = rng.integers(-1, d.n_nodes, 777).astype(np.int32)          # includes padding slots (-1)
    out = ctx.tgnn_gather_memory(graph, st, 1, dev(slots))
    o = Or.states[0]
    valid = slots >= 0; w = np.where(valid, slots, 0)
    me = np.where(valid, o["mail_eid"][w], -1); has = me >= 0
    assert np.array_equal(out["has_mail"].cpu().numpy(), has.astype(np.int32))
    assert np.array_equal(out["mem"].cpu().numpy(), (o["mem"][w] * valid[:, None]).astype(np.float32))
    assert np.array_equal(out["mail"].cpu().numpy(), (o["mail"][w] * valid[:, None]).astype(np.float32))
    assert np.array_equal(out["mail_efeat"].cpu().numpy(), P["efeat"][np.where(has, me, 0)] * has[:, None])
    assert np.array_equal(out["mem_ts"].cpu().numpy(), o["mem_ts"][w] * valid)
    assert np.array_equal(out["mail_ts"].cpu().numpy(), o["mail_ts"][w] * valid)
    # replica 0 of the device state is still all zero: its gather reports no mail anywhere
    out0 = ctx.tgnn_gather_memory(graph, st, 0, dev(slots))
    assert out0["has_mail"].sum().item() == 0 and out0["mem"].abs().sum().item() == 0

    params = tgnn.Params.from_numpy(P["params"])
    s_new, tau = ctx.tgnn_gru_update(params, out)
    # oracle on the float32-rounded state the device holds
    o32 = {k_: (v.astype(np.float32).astype(np.float64) if v.dtype == np.float64 and k_ in ("mem", "mail") else v)
           for k_, v in o.items()}
    ref_s, ref_tau, _ = O.updt_slots(o32, P["efeat"], Or.p, slots.astype(np.int64))
    assert np.array_equal(tau.cpu().numpy(), ref_tau)
    assert rel_err(s_new.cpu().numpy(), ref_s) <= TOL
    assert has.sum() > 50 and (~has & valid).sum() > 0 and np.abs(o["mem"]).max() > 0


@pytest.mark.parametrize("shape", [
    dict(R=500, k=10, d_m=100, d_s=0, d_e=172, d_t=100, H=2),
    dict(R=333, k=10, d_m=100, d_s=100, d_e=172, d_t=100, H=2),
    dict(R=64, k=5, d_m=24, d_s=6, d_e=0, d_t=10, H=3),
    dict(R=50, k=3, d_m=8, d_s=0, d_e=186, d_t=6, H=1),
])
def test_temporal_attention_fwd_bwd(shape):
    from paper_2307_07649_amd import tgnn
    R, k, d_m, d_s, d_e, d_t, H = (shape[n] for n in ("R", "k", "d_m", "d_s", "d_e", "d_t", "H"))
    d = synth.ModelDims(n_nodes=10, d_mem=d_m, d_time=d_t, d_edge=d_e, d_static=d_s, n_heads=H, k=k, batch=R)
    rng = np.random.default_rng(7)
    p32 = synth.gen_params(d, seed=3, random_phase=True)
    p = O.to_f64(p32)
    x_root = rng.standard_normal((R, d.d_x)).astype(np.float32)
    x_nbr = rng.standard_normal((R, k, d.d_x)).astype(np.float32)
    e_nbr = rng.standard_normal((R, k, d_e)).astype(np.float32)
    dt = rng.uniform(0, 3e5, (R, k))
    cnt = rng.integers(0, k + 1, R).astype(np.int32); cnt[:3] = [0, 1, k]
    dz = rng.standard_normal((R, d_m)).astype(np.float32)
    ctx = tgnn.Context(10, d_m, d_t, d_e, d_s, H, k, max_batch=(R + 2) // 3)
    params = tgnn.Params.from_numpy(p32); grads = tgnn.Params.zeros_like(params)
    z = ctx.tgnn_temporal_attn_fwd(params, dev(x_root), dev(x_nbr.reshape(R * k, -1)), dev(e_nbr.reshape(R * k, -1)),
                                   dev(dt.reshape(-1)), dev(cnt))
    mask = np.arange(k)[None] < cnt[:, None]
    zo, cache = O.attention_fwd(p, x_root.astype(np.float64), x_nbr * mask[..., None], e_nbr * mask[..., None],
                                dt * mask, cnt.astype(np.int64), H)
    assert rel_err(z.cpu().numpy(), zo) <= TOL
    d_root, d_nbr = ctx.tgnn_temporal_attn_bwd(params, dev(dz), grads)
    g, dxr, dxn = O.attention_bwd(p, cache, dz.astype(np.float64), H)
    assert rel_err(d_root.cpu().numpy(), dxr[:, :d_m]) <= TOL
    assert rel_err(d_nbr.cpu().numpy().reshape(R, k, d_m), dxn[:, :, :d_m] * mask[..., None]) <= TOL
    gg = grads.numpy()
    errs = {}
    for n in ("wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo", "time_w", "time_b"):      # each against its own largest entry
        # (the four tensors fed only by the score gradients: plus 16 fp32 roundings of their summed summand
        #  magnitudes -- the key bias is exactly zero in exact arithmetic; see gpu_common.compare_step)
        floor = 16 * FP32_EPS * float(cache["abs_terms"][n].max()) if n in cache["abs_terms"] else 0.0
        errs[n] = float(np.abs(gg[n] - g[n]).max() / (np.abs(g[n]).max() + floor / TOL))
    print(shape, {n: "%.2e" % v for n, v in errs.items()})
    assert all(v <= TOL for v in errs.values()), errs
    for n in ("gru_wih", "dec_ws", "dec_w2"):
        assert not gg[n].any()
    # a second backward call adds to the gradients (+= semantics)
    ctx.tgnn_temporal_attn_bwd(params, dev(dz), grads)
    assert rel_err(grads.numpy()["wv"], 2 * g["wv"]) <= TOL


def test_memory_writeback_last_event_wins():
    P = custom_problem(n_nodes=25, E=400, d_mem=100, d_time=8, d_edge=4, d_static=0, n_heads=2, k=5, batch=200)
    d = P["d"]
    tgnn, ctx, graph = make_ctx(P, n_replicas=3)
    rng = np.random.default_rng(5)
    st = tgnn.State(d.n_nodes, d.d_mem, 3)
    ost = O.new_state(d.n_nodes, d.d_mem)
    for rnd in range(3):                                        # consecutive calls reuse the arbitration scratch
        lo, hi = rnd * 130, rnd * 130 + 130 - rnd * 17
        b = batch_np(P, lo, hi); n = hi - lo
        s_src = rng.standard_normal((n, d.d_mem)).astype(np.float32); s_dst = rng.standard_normal((n, d.d_mem)).astype(np.float32)
        tau_s = rng.uniform(0, 50, n); tau_d = rng.uniform(0, 50, n)
        win = ctx.tgnn_memory_writeback(st, 2, dev(b["src"]), dev(b["dst"]), dev(b["eid"]), dev(b["t"]),
                                        dev(s_src), dev(s_dst), dev(tau_s), dev(tau_d))
        ow = O.writeback(ost, b["src"], b["dst"], b["eid"], b["t"], s_src.astype(np.float64), s_dst.astype(np.float64),
                         tau_s, tau_d)
        assert np.array_equal(win.cpu().numpy(), ow)
        N = d.n_nodes; s = slice(2 * N, 3 * N)
        assert np.array_equal(st.mem[s].cpu().numpy(), ost["mem"].astype(np.float32))
        assert np.array_equal(st.mail[s].cpu().numpy(), ost["mail"].astype(np.float32))
        assert np.array_equal(st.mail_eid[s].cpu().numpy(), ost["mail_eid"].astype(np.int32))
        assert np.array_equal(st.mail_ts[s].cpu().numpy(), ost["mail_ts"]) and np.array_equal(st.mem_ts[s].cpu().numpy(), ost["mem_ts"])
        assert st.mem[:2 * N].abs().sum().item() == 0 and (st.mail_eid[:2 * N] == -1).all().item()   # other replicas
    ctx.tgnn_state_reset(st, 2)
    assert st.mem.abs().sum().item() == 0 and (st.mail_eid == -1).all().item() and st.mail_ts.abs().sum().item() == 0


def test_error_paths_return_codes():
    P = custom_problem(n_nodes=30, E=100, d_mem=8, d_time=4, d_edge=2, d_static=0, n_heads=1, k=3, batch=10)
    tgnn, ctx, graph = make_ctx(P, n_replicas=2)
    import ctypes as C
    lib = tgnn._lib
    st = tgnn.State(30, 8, 2)
    assert lib.tgnn_state_reset(ctx.h, C.byref(st.c), 5, None) == -4
    qn = dev(np.zeros(8, np.int32)); qt = dev(np.zeros(8))
    assert lib.tgnn_sample_recent(ctx.h, C.byref(graph.c), qn.data_ptr(), qt.data_ptr(), 8, None, None, None, None, None) == -2
    assert b"NULL" in lib.tgnn_last_error()
    assert lib.tgnn_sample_recent(ctx.h, C.byref(graph.c), qn.data_ptr() + 4, qt.data_ptr(), 4, qn.data_ptr(), qn.data_ptr(),
                                  qt.data_ptr(), qn.data_ptr(), None) == -3
    params = tgnn.Params.from_numpy(P["params"]); grads = tgnn.Params.zeros_like(params)
    loss = torch.zeros(4, device="cuda")
    b = batch_np(P, 0, 10)
    ok = tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"], replica=0)
    dup = tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"], replica=0)
    with pytest.raises(tgnn.TgnnError) as e:
        ctx.tgnn_train_step(graph, st, params, grads, [ok, dup], out_loss=loss)
    assert e.value.code == -1
    big = batch_np(P, 0, 11)
    with pytest.raises(tgnn.TgnnError) as e:
        ctx.tgnn_train_step(graph, st, params, grads, [tgnn.Batch(big["src"], big["dst"], big["neg"], big["eid"], big["t"])],
                            out_loss=loss)
    assert e.value.code == -4
    with pytest.raises(tgnn.TgnnError) as e:
        ctx.tgnn_train_step(graph, st, params, grads, [tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"], replica=2)],
                            out_loss=loss)
    assert e.value.code == -4
    # an empty batch is legal: loss 0, nothing written
    empty = batch_np(P, 0, 0)
    ctx.tgnn_train_step(graph, st, params, grads, [tgnn.Batch(empty["src"], empty["dst"], empty["neg"], empty["eid"], empty["t"])],
                        out_loss=loss)
    torch.cuda.synchronize()
    assert loss[0].item() == 0 and (st.mail_eid == -1).all().item()
