"""CPU oracle for the memory-based TGNN training step (TGN-attn with static node memory).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP path is
compared against.  Only tests, the smoke check and the benchmark's cpu-baseline leg may use
it; the product path never does.  It shares no code with the HIP library, and it imports
nothing but numpy.  All floating point is float64.

What each function follows (paper = DistTGL, arXiv 2307.07649):
  * events (u, v, e_uv, t), zero-initialised node memory s_v, mails
    m_u = {s_u || s_v || Phi(t - t_u^-) || e_uv}                      -- Sec. 2.1, Eq. 1-2
  * s_u = UPDT(s_u, m_u) with UPDT a GRU cell, no gradient into earlier cells -- Eq. 3, Sec. 2.1
  * one-layer temporal attention over the most recent neighbours   -- Eq. 4-7
  * mails cached, embeddings computed before the memory is written ("reversed
    computation order"); COMB keeps the most recent mail of a batch -- Sec. 2.1, 2.1.1, Eq. 8
  * memory and mails fetched for root and supporting nodes, UPDT re-computed for
    supporting nodes, only root nodes written back                 -- Sec. 3.2.1
  * static node memory combined with the dynamic memory            -- Sec. 3.1
  * self-supervision by temporal edges with sampled negative destinations -- Sec. 2.1, 3.2.2
  * memory and mails reset at the start of an epoch                -- Alg. 1

Where the paper is silent the readings are (they are listed with reasons in the design notes):
  undirected neighbour lists ordered by (time, event id); "most recent" = time strictly
  below the query time; Phi(d)_c = cos(w_c d + b_c) evaluated in double; the usual GRU cell
  (gates r, z, n; reset gate applied to W_hn h + b_hn); the time difference in the keys is
  query time minus the update time of the neighbour's memory as used (option: minus the edge
  time); softmax scale 1/sqrt(|N_v|); heads are contiguous slices; merge layer
  z = ReLU(W_o {h_v || x_v} + b_o); decoder logit = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2;
  loss = mean binary cross-entropy over B positive and B negative pairs; a mail row stores
  {s'_self || s'_other} and the event id, Phi and e_uv are looked up when the mail is consumed.

Parity pins (tests/test_oracle_*.py): brute-force neighbour scan, closed forms of the time
encoding, a library GRU cell and its limits, attention special cases, ln 2 loss, central
finite differences for every parameter tensor, brute-force last-writer-wins write-back.
The step as a whole is "parity unpinned" against the paper, which prints no worked example.
"""
from __future__ import annotations

import numpy as np

F = np.float64

PARAM_NAMES = ["time_w", "time_b", "gru_wih", "gru_whh", "gru_bih", "gru_bhh", "wq", "bq", "wk", "bk",
               "wv", "bv", "wo", "bo", "dec_ws", "dec_wd", "dec_b1", "dec_w2", "dec_b2"]
FROZEN_IN_SGD = ("time_w", "time_b")


# --------------------------------------------------------------------------------------
# state
# --------------------------------------------------------------------------------------
def new_state(n_nodes: int, d_mem: int):
    """All-zero memory and mailbox: the state at the start of every epoch (Alg. 1, 'reset')."""
    return dict(mem=np.zeros((n_nodes, d_mem), F), mem_ts=np.zeros(n_nodes, F),
                mail=np.zeros((n_nodes, 2 * d_mem), F), mail_ts=np.zeros(n_nodes, F),
                mail_eid=np.full(n_nodes, -1, np.int64))


def to_f64(params):
    return {k: np.asarray(v, dtype=F).copy() for k, v in params.items()}


# --------------------------------------------------------------------------------------
# most-recent-neighbour sampling (Sec. 2.1: "most recent neighbors"; k = 10 in Sec. 4)
# --------------------------------------------------------------------------------------
def build_adjacency(src, dst, ts, n_nodes):
    """Every event is incident to both endpoints.  Per node, incident events ordered by
    (time, event id).  Returns (indptr, other, eid, time) in that order."""
    src = np.asarray(src, np.int64); dst = np.asarray(dst, np.int64); ts = np.asarray(ts, F)
    E = src.shape[0]
    node = np.concatenate([src, dst]); other = np.concatenate([dst, src])
    eid = np.concatenate([np.arange(E), np.arange(E)]); tt = np.concatenate([ts, ts])
    order = np.lexsort((eid, tt, node))          # primary key node, then time, then event id
    node, other, eid, tt = node[order], other[order], eid[order], tt[order]
    indptr = np.zeros(n_nodes + 1, np.int64)
    np.add.at(indptr, node + 1, 1)
    indptr = np.cumsum(indptr)
    return indptr, other, eid, tt


def sample_recent(adj, q_node, q_t, k):
    """For each query (node, t): the min(k, #) incident events with time strictly below t that come
    last in (time, event id) order, listed most recent first.  Padding: nbr = eid = -1, time = 0."""
    indptr, other, eid, tt = adj
    R = len(q_node)
    nbr = np.full((R, k), -1, np.int64); ne = np.full((R, k), -1, np.int64)
    nts = np.zeros((R, k), F); cnt = np.zeros(R, np.int64)
    for r in range(R):
        lo, hi = indptr[q_node[r]], indptr[q_node[r] + 1]
        pos = lo + np.searchsorted(tt[lo:hi], q_t[r], side="left")     # first entry with time >= t
        c = min(k, pos - lo)
        sel = pos - 1 - np.arange(c)
        nbr[r, :c] = other[sel]; ne[r, :c] = eid[sel]; nts[r, :c] = tt[sel]; cnt[r] = c
    return nbr, ne, nts, cnt


# --------------------------------------------------------------------------------------
# time encoding Phi (Eq. 1-2, 5-6)
# --------------------------------------------------------------------------------------
def time_encode(delta, w, b):
    """Phi(delta)_c = cos(w_c * delta + b_c).  delta: [...]; returns [..., d_time]."""
    delta = np.asarray(delta, F)
    return np.cos(delta[..., None] * w + b)


# --------------------------------------------------------------------------------------
# GRU cell = UPDT (Eq. 3)
# --------------------------------------------------------------------------------------
def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def gru_cell(x, h, wih, whh, bih, bhh, want_cache=False):
    d = h.shape[-1]
    gi = x @ wih.T + bih
    gh = h @ whh.T + bhh
    r = _sigmoid(gi[..., :d] + gh[..., :d])
    z = _sigmoid(gi[..., d:2 * d] + gh[..., d:2 * d])
    hn = gh[..., 2 * d:]
    n = np.tanh(gi[..., 2 * d:] + r * hn)
    out = (1.0 - z) * n + z * h
    if want_cache:
        return out, dict(r=r, z=z, n=n, hn=hn)
    return out


def updt_slots(state, efeat, p, slot_node):
    """UPDT for every slot node from the stored (pre-batch) state (Sec. 2.1.1, 3.2.1):
    a node with a cached mail gets s' = GRU({mail || Phi(mail_ts - mem_ts) || e_mail}, s), tau = mail_ts;
    a node without one keeps s' = s, tau = mem_ts.  slot_node = -1 marks padding (all zeros)."""
    valid = slot_node >= 0
    w = np.where(valid, slot_node, 0)
    me = state["mail_eid"][w]
    has = valid & (me >= 0)
    delta = np.where(has, state["mail_ts"][w] - state["mem_ts"][w], 0.0)
    arg = delta[:, None] * p["time_w"] + p["time_b"]
    phi = np.cos(arg)
    d_e = efeat.shape[1]
    ef = efeat[np.where(has, me, 0)].astype(F) if d_e else np.zeros((len(w), 0), F)
    x = np.concatenate([state["mail"][w], phi, ef], axis=1)
    h = state["mem"][w]
    hnew, c = gru_cell(x, h, p["gru_wih"], p["gru_whh"], p["gru_bih"], p["gru_bhh"], want_cache=True)
    s_new = np.where(has[:, None], hnew, h) * valid[:, None]
    tau = np.where(has, state["mail_ts"][w], state["mem_ts"][w]) * valid
    c.update(x=x, h=h, has=has, delta=delta, arg=arg)
    return s_new, tau, c


# --------------------------------------------------------------------------------------
# temporal attention (Eq. 4-7) + merge layer
# --------------------------------------------------------------------------------------
def attention_fwd(p, x_root, x_nbr, e_nbr, dt_nbr, cnt, n_heads):
    """x_root [R, d_x]; x_nbr [R, k, d_x]; e_nbr [R, k, d_e]; dt_nbr [R, k]; cnt [R].
    q = W_q {x_v || Phi(0)} + b_q;  K, V = W {x_w || e_vw || Phi(dt)} + b;
    per head: softmax_j(q . K_j / sqrt(cnt)) V over the cnt valid neighbours (0 if none);
    z = ReLU(W_o {h_v || x_v} + b_o)."""
    R, k, _ = x_nbr.shape
    d_o = p["wq"].shape[0]
    phi0 = np.broadcast_to(np.cos(p["time_b"]), (R, p["time_b"].shape[0]))
    q_in = np.concatenate([x_root, phi0], axis=1)
    q = q_in @ p["wq"].T + p["bq"]
    arg = dt_nbr[..., None] * p["time_w"] + p["time_b"]
    c_in = np.concatenate([x_nbr, e_nbr, np.cos(arg)], axis=2)
    K = c_in @ p["wk"].T + p["bk"]
    V = c_in @ p["wv"].T + p["bv"]
    mask = np.arange(k)[None, :] < cnt[:, None]
    dh = d_o // n_heads
    scale = 1.0 / np.sqrt(np.maximum(cnt, 1).astype(F))
    qh = q.reshape(R, n_heads, dh); Kh = K.reshape(R, k, n_heads, dh); Vh = V.reshape(R, k, n_heads, dh)
    a = np.einsum("rhd,rjhd->rhj", qh, Kh) * scale[:, None, None]
    a = np.where(mask[:, None, :], a, -np.inf)
    amax = np.max(a, axis=2, keepdims=True)
    amax = np.where(np.isfinite(amax), amax, 0.0)
    ex = np.where(mask[:, None, :], np.exp(a - amax), 0.0)
    den = ex.sum(axis=2, keepdims=True)
    pr = np.where(den > 0, ex / np.where(den > 0, den, 1.0), 0.0)          # [R, H, k]
    o = np.einsum("rhj,rjhd->rhd", pr, Vh).reshape(R, d_o)
    m_in = np.concatenate([o, x_root], axis=1)
    zpre = m_in @ p["wo"].T + p["bo"]
    z = np.maximum(zpre, 0.0)
    cache = dict(q_in=q_in, q=q, c_in=c_in, arg=arg, K=K, V=V, pr=pr, scale=scale, mask=mask, o=o,
                 m_in=m_in, zpre=zpre, dt=dt_nbr)
    return z, cache


def attention_bwd(p, cache, dz, n_heads):
    """Reverse mode through attention_fwd.  Returns (param grads, d x_root, d x_nbr)."""
    g = {}
    q_in, c_in, K, V, pr, scale, mask = (cache[n] for n in ("q_in", "c_in", "K", "V", "pr", "scale", "mask"))
    R, k, d_kv = c_in.shape
    d_o = p["wq"].shape[0]; dh = d_o // n_heads
    d_x = q_in.shape[1] - p["time_b"].shape[0]
    dzpre = dz * (cache["zpre"] > 0)
    g["wo"] = dzpre.T @ cache["m_in"]; g["bo"] = dzpre.sum(0)
    dm_in = dzpre @ p["wo"]
    do = dm_in[:, :d_o]; dx_root = dm_in[:, d_o:].copy()
    doh = do.reshape(R, n_heads, dh)
    Vh = V.reshape(R, k, n_heads, dh); Kh = K.reshape(R, k, n_heads, dh); qh = cache["q"].reshape(R, n_heads, dh)
    dpr = np.einsum("rhd,rjhd->rhj", doh, Vh)
    dVh = np.einsum("rhj,rhd->rjhd", pr, doh)
    da = pr * (dpr - (pr * dpr).sum(axis=2, keepdims=True))
    da = da * scale[:, None, None]
    dqh = np.einsum("rhj,rjhd->rhd", da, Kh)
    dKh = np.einsum("rhj,rhd->rjhd", da, qh)
    dq = dqh.reshape(R, d_o); dK = dKh.reshape(R, k, d_o); dV = dVh.reshape(R, k, d_o)
    mk = mask[..., None]
    dK = dK * mk; dV = dV * mk
    cf = c_in.reshape(R * k, d_kv) * mask.reshape(R * k, 1)
    g["wk"] = dK.reshape(R * k, d_o).T @ cf; g["bk"] = dK.sum((0, 1))
    g["wv"] = dV.reshape(R * k, d_o).T @ cf; g["bv"] = dV.sum((0, 1))
    dc = dK @ p["wk"] + dV @ p["wv"]                         # [R, k, d_kv]
    dx_nbr = dc[:, :, :d_x]
    dphi = dc[:, :, d_kv - p["time_b"].shape[0]:] * mk
    msin = -np.sin(cache["arg"])
    g["time_w"] = (dphi * msin * cache["dt"][..., None]).sum((0, 1))
    g["time_b"] = (dphi * msin).sum((0, 1))
    g["wq"] = dq.T @ q_in; g["bq"] = dq.sum(0)
    dq_in = dq @ p["wq"]
    dx_root += dq_in[:, :d_x]
    g["time_b"] = g["time_b"] + (dq_in[:, d_x:] * (-np.sin(p["time_b"]))).sum(0)   # Phi(0): d/dw = 0
    return g, dx_root, dx_nbr


# --------------------------------------------------------------------------------------
# link-prediction decoder + binary cross-entropy
# --------------------------------------------------------------------------------------
def _softplus(x):
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def decoder_loss(p, z_src, z_dst, z_neg):
    """logit(a, b) = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2 for the B true pairs and the B pairs with a
    sampled negative destination; loss = mean of softplus(-logit+) and softplus(logit-) over 2B."""
    B = z_src.shape[0]
    a = np.concatenate([z_src, z_src], 0); b = np.concatenate([z_dst, z_neg], 0)
    hpre = a @ p["dec_ws"].T + b @ p["dec_wd"].T + p["dec_b1"]
    h1 = np.maximum(hpre, 0.0)
    logits = h1 @ p["dec_w2"] + p["dec_b2"][0]
    y = np.concatenate([np.ones(B), np.zeros(B)])
    loss = (_softplus(-logits[:B]).sum() + _softplus(logits[B:]).sum()) / (2 * B) if B else 0.0
    return loss, logits, dict(a=a, b=b, hpre=hpre, h1=h1, y=y)


def decoder_bwd(p, cache, logits, loss_scale=1.0):
    B2 = logits.shape[0]; B = B2 // 2
    g = {}
    dl = (_sigmoid(logits) - cache["y"]) / B2 * loss_scale
    g["dec_w2"] = cache["h1"].T @ dl; g["dec_b2"] = np.array([dl.sum()])
    dh = dl[:, None] * p["dec_w2"][None, :] * (cache["hpre"] > 0)
    g["dec_ws"] = dh.T @ cache["a"]; g["dec_wd"] = dh.T @ cache["b"]; g["dec_b1"] = dh.sum(0)
    da = dh @ p["dec_ws"]; db = dh @ p["dec_wd"]
    return g, da[:B] + da[B:], db[:B], db[B:]


# --------------------------------------------------------------------------------------
# last-event-wins write-back (COMB = most recent mail, Eq. 8; roots only, Sec. 3.2.1)
# --------------------------------------------------------------------------------------
def writeback(state, src, dst, eid, t, s_src, s_dst, tau_src, tau_dst):
    """Walk the batch in event order; within an event the source is written first, then the
    destination, so the occurrence with the largest (event index, role) wins for each node.
    Returns winner flags indexed [role * B + i]."""
    B = len(src)
    last = {}
    for i in range(B):
        last[int(src[i])] = (i, 0)
        last[int(dst[i])] = (i, 1)
    win = np.zeros(2 * B, np.int32)
    for node, (i, role) in last.items():
        win[role * B + i] = 1
        s_self, s_oth = (s_src[i], s_dst[i]) if role == 0 else (s_dst[i], s_src[i])
        state["mem"][node] = s_self
        state["mem_ts"][node] = tau_src[i] if role == 0 else tau_dst[i]
        state["mail"][node] = np.concatenate([s_self, s_oth])
        state["mail_eid"][node] = eid[i]
        state["mail_ts"][node] = t[i]
    return win


# --------------------------------------------------------------------------------------
# one training step on one mini-batch
# --------------------------------------------------------------------------------------
def forward_backward(state, adj, efeat, static, p, batch, k, n_heads, dt_source=0, loss_scale=1.0,
                     want_grads=True):
    """batch = dict(src, dst, neg, eid, t).  Returns dict(loss, logits, grads, nbr, neid, nts, cnt,
    s_new, tau, z).  Does not modify `state`."""
    src, dst, neg = (np.asarray(batch[n], np.int64) for n in ("src", "dst", "neg"))
    t = np.asarray(batch["t"], F)
    B = len(src); R = 3 * B
    d_m = state["mem"].shape[1]; d_t = p["time_w"].shape[0]
    root_node = np.concatenate([src, dst, neg]); root_t = np.concatenate([t, t, t])
    nbr, neid, nts, cnt = sample_recent(adj, root_node, root_t, k)
    slot_node = np.concatenate([root_node, nbr.reshape(-1)])
    s_new, tau, gc = updt_slots(state, efeat, p, slot_node)

    def with_static(nodes, s):
        if static is None:
            return s
        st = static[np.where(nodes >= 0, nodes, 0)].astype(F) * (nodes >= 0)[..., None]
        return np.concatenate([s, st], axis=-1)

    x_root = with_static(root_node, s_new[:R])
    x_nbr = with_static(nbr, s_new[R:].reshape(R, k, d_m))
    valid = nbr >= 0
    e_nbr = efeat[np.where(valid, neid, 0)].astype(F) * valid[..., None]
    ref_t = tau[R:].reshape(R, k) if dt_source == 0 else nts
    dt_nbr = np.where(valid, root_t[:, None] - ref_t, 0.0)
    z, ac = attention_fwd(p, x_root, x_nbr, e_nbr, dt_nbr, cnt, n_heads)
    loss, logits, dc = decoder_loss(p, z[:B], z[B:2 * B], z[2 * B:])
    out = dict(loss=loss, logits=logits, nbr=nbr, neid=neid, nts=nts, cnt=cnt, s_new=s_new, tau=tau, z=z,
               dt_nbr=dt_nbr, zpre=ac["zpre"], hpre=dc["hpre"])
    if not want_grads:
        return out

    g, dzs, dzd, dzn = decoder_bwd(p, dc, logits, loss_scale)
    ga, dx_root, dx_nbr = attention_bwd(p, ac, np.concatenate([dzs, dzd, dzn], 0), n_heads)
    g.update(ga)
    # gradient reaching s' of every slot; it stops at the stored memory and mails (no BPTT)
    ds = np.concatenate([dx_root[:, :d_m], dx_nbr[:, :, :d_m].reshape(R * k, d_m)], 0)
    ds = ds * gc["has"][:, None]
    r, zg, n, hn, h, x = (gc[nm] for nm in ("r", "z", "n", "hn", "h", "x"))
    dn = ds * (1.0 - zg); dzg = ds * (h - n)
    dnpre = dn * (1.0 - n * n)
    dr = dnpre * hn
    dzpre = dzg * zg * (1.0 - zg); drpre = dr * r * (1.0 - r)
    dgi = np.concatenate([drpre, dzpre, dnpre], 1)
    dgh = np.concatenate([drpre, dzpre, dnpre * r], 1)
    g["gru_wih"] = dgi.T @ x; g["gru_bih"] = dgi.sum(0)
    g["gru_whh"] = dgh.T @ h; g["gru_bhh"] = dgh.sum(0)
    dphi = (dgi @ p["gru_wih"])[:, 2 * d_m:2 * d_m + d_t]
    msin = -np.sin(gc["arg"])
    g["time_w"] = g["time_w"] + (dphi * msin * gc["delta"][:, None]).sum(0)
    g["time_b"] = g["time_b"] + (dphi * msin).sum(0)
    out["grads"] = {n: g[n] for n in PARAM_NAMES}
    return out


def apply_writeback(state, batch, fb):
    B = len(batch["src"])
    return writeback(state, batch["src"], batch["dst"], batch["eid"], batch["t"],
                     fb["s_new"][:B], fb["s_new"][B:2 * B], fb["tau"][:B], fb["tau"][B:2 * B])


def sgd(p, grads, lr):
    """Plain SGD on every tensor except the time-encoding frequencies and phases."""
    for n in PARAM_NAMES:
        if n not in FROZEN_IN_SGD:
            p[n] -= lr * grads[n]


def train_step(states, adj, efeat, static, p, batches, k, n_heads, lr=0.0, dt_source=0):
    """One step over len(batches) memory replicas that share one weight set (memory parallelism,
    Sec. 3.2.3): replica i advances states[i] on batches[i]; gradients are summed, the loss is the
    mean of the per-batch losses; then one SGD update and the write-backs."""
    outs = [forward_backward(states[i], adj, efeat, static, p, batches[i], k, n_heads, dt_source)
            for i in range(len(batches))]
    grads = {n: sum(o["grads"][n] for o in outs) for n in PARAM_NAMES}
    loss = float(np.mean([o["loss"] for o in outs]))
    wins = [apply_writeback(states[i], batches[i], outs[i]) for i in range(len(batches))]
    if lr:
        sgd(p, grads, lr)
    return dict(loss=loss, grads=grads, outs=outs, winners=wins)
