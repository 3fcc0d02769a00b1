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
  * dynamic edge classification with C classes and multi-label targets (the GDELT task)
    and the mean reciprocal rank of the true destination among 49 sampled ones; the counts behind
    the micro-averaged F1 score                                     -- Sec. 4 "Datasets"

Where the paper is silent the readings are (they are listed with reasons in the design notes):
  undirected neighbour lists ordered by (time, event id); "most recent" = time strictly
  below the query time; Phi(d)_c = cos(w_c d + b_c) evaluated in double; the usual GRU cell
  (gates r, z, n; reset gate applied to W_hn h + b_hn); the time difference in the keys is
  query time minus the update time of the neighbour's memory as used (option: minus the edge
  time); softmax scale 1/sqrt(|N_v|); heads are contiguous slices; merge layer
  z = ReLU(W_o {h_v || x_v} + b_o); decoder logit = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2;
  loss = mean binary cross-entropy over B positive and B negative pairs; a mail row stores
  {s'_self || s'_other} and the event id, Phi and e_uv are looked up when the mail is consumed.

Parity pins (tests/test_oracle_*.py): hand-written neighbour lists and a pure-Python event scan
for the sampler (and the indexed form against the scan); closed forms of the time encoding, on the
function and on the values the step feeds to the GRU, the keys and the query (hand-built states
with known time differences and non-zero phases); a library GRU cell and its limits; attention
special cases; ln 2 loss; central finite differences for every parameter tensor; brute-force
last-writer-wins write-back; the classification head: ln 2 at zero weights, a hand-computed event, finite
differences; the reciprocal rank: hand-written score lists with ties; the F1 counts: a hand-written table.
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
def sample_recent(src, dst, ts, q_node, q_t, k):
    """The definition, as a scan of the raw chronological event list.  Every event (u, v, t) is incident
    to both endpoints; for a query (node, t_q) the candidates are the incident events with time strictly
    below t_q, ordered by (time, event id); the last min(k, #) of them are returned, most recent first.
    An event with u = v = node is incident to the node once as a source and once as a destination, so it
    is listed twice.  Padding: nbr = eid = -1, time = 0.
    src, dst, ts: the whole event list, ts non-decreasing (then event-id order is (time, id) order)."""
    src = np.asarray(src, np.int64); dst = np.asarray(dst, np.int64); ts = np.asarray(ts, F)
    R = len(q_node)
    nbr = np.full((R, k), -1, np.int64); ne = np.full((R, k), -1, np.int64)
    nts = np.zeros((R, k), F); cnt = np.zeros(R, np.int64)
    for r in range(R):
        v = q_node[r]
        as_src = np.flatnonzero(src == v)                     # events leaving v: the other endpoint is dst
        as_dst = np.flatnonzero(dst == v)                     # events entering v: the other endpoint is src
        e = np.concatenate([as_src, as_dst])
        other = np.concatenate([dst[as_src], src[as_dst]])
        keep = ts[e] < q_t[r]                                 # strictly earlier than the query
        e, other = e[keep], other[keep]
        order = np.argsort(e, kind="stable")                  # (time, event id) order = event-id order
        e, other = e[order], other[order]
        c = min(k, len(e))
        if c:
            nbr[r, :c] = other[::-1][:c]; ne[r, :c] = e[::-1][:c]; nts[r, :c] = ts[e[::-1][:c]]
        cnt[r] = c
    return nbr, ne, nts, cnt


def build_adjacency(src, dst, ts, n_nodes):
    """Per-node lists of incident events ordered by (time, event id): an index over the event list for
    graphs on which the scan above would take hours.  Returns (indptr, other, eid, time)."""
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


def sample_recent_indexed(adj, q_node, q_t, k):
    """Same result as sample_recent, read off the per-node lists of build_adjacency (the tests hold the
    two against each other).  Used only where the event list is too long to scan once per query."""
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


def event_list(src, dst, ts):
    """The graph argument of forward_backward / train_step: the raw event list (neighbours by scan)."""
    return dict(src=np.asarray(src, np.int64), dst=np.asarray(dst, np.int64), ts=np.asarray(ts, F))


# --------------------------------------------------------------------------------------
# time encoding Phi (Eq. 1-2, 5-6)
# --------------------------------------------------------------------------------------
def time_encode(delta, w, b):
    """Phi(delta)_c = cos(w_c * delta + b_c).  delta: [...]; returns [..., d_time]."""
    delta = np.asarray(delta, F)
    return np.cos(delta[..., None] * w + b)


def time_encode_darg(delta, w, b):
    """d Phi(delta)_c / d(w_c delta + b_c) = -sin(w_c delta + b_c): what the backward pass multiplies by
    (times delta for the gradient of w_c, times 1 for that of b_c)."""
    delta = np.asarray(delta, F)
    return -np.sin(delta[..., None] * w + b)


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
    phi = time_encode(delta, p["time_w"], p["time_b"])
    d_e = efeat.shape[1]
    ef = efeat[np.where(has, me, 0)].astype(F) if d_e else np.zeros((len(w), 0), F)
    x = np.concatenate([state["mail"][w], phi, ef], axis=1)
    h = state["mem"][w]
    hnew, c = gru_cell(x, h, p["gru_wih"], p["gru_whh"], p["gru_bih"], p["gru_bhh"], want_cache=True)
    s_new = np.where(has[:, None], hnew, h) * valid[:, None]
    tau = np.where(has, state["mail_ts"][w], state["mem_ts"][w]) * valid
    c.update(x=x, h=h, has=has, delta=delta)
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
    phi0 = time_encode(np.zeros(R), p["time_w"], p["time_b"])          # the query's own time difference is 0
    q_in = np.concatenate([x_root, phi0], axis=1)
    q = q_in @ p["wq"].T + p["bq"]
    c_in = np.concatenate([x_nbr, e_nbr, time_encode(dt_nbr, p["time_w"], p["time_b"])], axis=2)
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
    cache = dict(q_in=q_in, q=q, c_in=c_in, K=K, V=V, pr=pr, scale=scale, mask=mask, o=o,
                 m_in=m_in, zpre=zpre, dt=dt_nbr)
    return z, cache


def attention_bwd(p, cache, dz, n_heads, gate_z=None):
    """Reverse mode through attention_fwd.  Returns (param grads, d x_root, d x_nbr).
    gate_z (bool [R, d_o], optional): the ReLU gate of the merge layer to differentiate through instead of
    zpre > 0 -- for a comparison with an implementation that decided a pre-activation within rounding of zero
    the other way (the decision is then taken once, in that implementation's precision)."""
    g = {}
    q_in, c_in, K, V, pr, scale, mask = (cache[n] for n in ("q_in", "c_in", "K", "V", "pr", "scale", "mask"))
    R, k, d_kv = c_in.shape
    d_o = p["wq"].shape[0]; dh = d_o // n_heads
    d_x = q_in.shape[1] - p["time_b"].shape[0]
    dzpre = dz * ((cache["zpre"] > 0) if gate_z is None else gate_z)
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
    # Not gradients: for the four tensors fed by the score gradients da only, the same sums over magnitudes, with
    # |da| taken before the cancellation inside the softmax's backward pass, pr (|dpr| + sum pr |dpr|).  The softmax is
    # invariant to a shift of all scores of a root, so the exact gradient of bk is zero, and with identical keys
    # those of wq, bq, wk vanish too; these sums are the scale the rounding error of such a result lives on.
    da_mag = pr * (np.abs(dpr) + (pr * np.abs(dpr)).sum(axis=2, keepdims=True)) * scale[:, None, None]
    dq_mag = np.einsum("rhj,rjhd->rhd", da_mag, np.abs(Kh)).reshape(R, d_o)
    dK_mag = np.einsum("rhj,rhd->rjhd", da_mag, np.abs(qh)).reshape(R, k, d_o) * mk
    cache["abs_terms"] = dict(wq=dq_mag.T @ np.abs(q_in), bq=dq_mag.sum(0),
                              wk=dK_mag.reshape(R * k, d_o).T @ np.abs(cf), bk=dK_mag.sum((0, 1)))
    g["wv"] = dV.reshape(R * k, d_o).T @ cf; g["bv"] = dV.sum((0, 1))
    dc = dK @ p["wk"] + dV @ p["wv"]                         # [R, k, d_kv]
    dx_nbr = dc[:, :, :d_x]
    dphi = dc[:, :, d_kv - p["time_b"].shape[0]:] * mk
    msin = time_encode_darg(cache["dt"], p["time_w"], p["time_b"])
    g["time_w"] = (dphi * msin * cache["dt"][..., None]).sum((0, 1))
    g["time_b"] = (dphi * msin).sum((0, 1))
    g["wq"] = dq.T @ q_in; g["bq"] = dq.sum(0)
    dq_in = dq @ p["wq"]
    dx_root += dq_in[:, :d_x]
    g["time_b"] = g["time_b"] + (dq_in[:, d_x:] * time_encode_darg(np.zeros(R), p["time_w"], p["time_b"])).sum(0)
    # (Phi(0) does not depend on w)
    return g, dx_root, dx_nbr


# --------------------------------------------------------------------------------------
# link-prediction decoder + binary cross-entropy
# --------------------------------------------------------------------------------------
def _softplus(x):
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def decoder_loss(p, z_src, z_dst, z_neg):
    """logit(a, b) = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2 for the B true pairs and the B pairs with a
    sampled negative destination; loss = mean of softplus(-logit+) and softplus(logit-) over 2B.
    z_neg may hold J sets of B negative destinations, [J B, d] (epoch parallelism, Sec. 3.2.2: J trainers share the
    positive batch and differ in their negatives): logits are [B true | B per set], the loss is the mean over the
    sets of each set's loss (the true pairs belong to every set)."""
    B = z_src.shape[0]
    J = z_neg.shape[0] // B if B else 1
    a = np.concatenate([z_src] * (1 + J), 0); b = np.concatenate([z_dst, z_neg], 0)
    hpre = a @ p["dec_ws"].T + b @ p["dec_wd"].T + p["dec_b1"]
    h1 = np.maximum(hpre, 0.0)
    logits = h1 @ p["dec_w2"] + p["dec_b2"][0]
    y = np.concatenate([np.ones(B), np.zeros(J * B)])
    loss = (_softplus(-logits[:B]).sum() + _softplus(logits[B:]).sum() / J) / (2 * B) if B else 0.0
    return loss, logits, dict(a=a, b=b, hpre=hpre, h1=h1, y=y, J=J)


def decoder_bwd(p, cache, logits, loss_scale=1.0, gate_h=None):
    """gate_h (bool [2B, d_o], optional): the ReLU gate of the hidden layer to use instead of hpre > 0 (see
    attention_bwd)."""
    J = cache["J"]; B = logits.shape[0] // (1 + J)
    g = {}
    # gradient of the SUM of the J sets' losses (each a mean over its 2B pairs): a true pair is in every set
    dl = (_sigmoid(logits) - cache["y"]) / (2 * B) * loss_scale
    dl[:B] *= J
    g["dec_w2"] = cache["h1"].T @ dl; g["dec_b2"] = np.array([dl.sum()])
    dh = dl[:, None] * p["dec_w2"][None, :] * ((cache["hpre"] > 0) if gate_h is None else gate_h)
    g["dec_ws"] = dh.T @ cache["a"]; g["dec_wd"] = dh.T @ cache["b"]; g["dec_b1"] = dh.sum(0)
    da = dh @ p["dec_ws"]; db = dh @ p["dec_wd"]
    return g, da.reshape(1 + J, B, da.shape[1]).sum(0), db[:B], db[B:]


def edge_class_loss(p, z_src, z_dst, labels):
    """Dynamic edge classification (Sec. 4 "Datasets": C classes, several of them true for an event): the
    decoder's hidden layer as in decoder_loss, C outputs logit_c = W2[c] . ReLU(W_s z_src + W_d z_dst + b1) + b2[c]
    (dec_w2 is [C, d_o], dec_b2 [C]); labels [B, C] in {0, 1}; loss = mean over the B events and the C classes of the
    binary cross-entropy softplus(logit) - y logit."""
    hpre = z_src @ p["dec_ws"].T + z_dst @ p["dec_wd"].T + p["dec_b1"]
    h1 = np.maximum(hpre, 0.0)
    logits = h1 @ p["dec_w2"].T + p["dec_b2"]
    y = np.asarray(labels, F)
    loss = float((_softplus(logits) - y * logits).mean()) if logits.size else 0.0
    return loss, logits, dict(a=z_src, b=z_dst, hpre=hpre, h1=h1, y=y)


def edge_class_bwd(p, cache, logits, loss_scale=1.0, gate_h=None):
    """Gradients of edge_class_loss; returns (weight gradients, dz_src, dz_dst)."""
    B, C = logits.shape
    g = {}
    dl = (_sigmoid(logits) - cache["y"]) / (B * C) * loss_scale
    g["dec_w2"] = dl.T @ cache["h1"]; g["dec_b2"] = dl.sum(0)
    dh = (dl @ p["dec_w2"]) * ((cache["hpre"] > 0) if gate_h is None else gate_h)
    g["dec_ws"] = dh.T @ cache["a"]; g["dec_wd"] = dh.T @ cache["b"]; g["dec_b1"] = dh.sum(0)
    return g, dh @ p["dec_ws"], dh @ p["dec_wd"]


def f1_micro_counts(logits, labels):
    """Counts behind the micro-averaged F1 score of the edge-classification task (Sec. 4: "we report the F1-Micro
    score"): a class is predicted for an event when its logit is positive (probability above one half); over all
    events and classes, tp = predicted and true, fp = predicted and not true, fn = true and not predicted.
    F1-micro = 2 tp / (2 tp + fp + fn).  Returns (tp, fp, fn)."""
    pred = np.asarray(logits) > 0
    y = np.asarray(labels) > 0.5
    return int((pred & y).sum()), int((pred & ~y).sum()), int((~pred & y).sum())


def reciprocal_rank(score_true, score_neg):
    """Rank of the true destination among itself and the sampled negative destinations of its event (Sec. 4: 49 of
    them, mean reciprocal rank reported).  score_true [B], score_neg [J, B].  rank = 1 + the number of negatives
    that score strictly higher + half the number that score exactly the same (the expected rank when ties are broken
    at random; the paper does not say how it breaks them).  Returns (rank [B], mean of 1 / rank)."""
    st = np.asarray(score_true, F); sn = np.asarray(score_neg, F).reshape(-1, len(st))
    rank = 1.0 + (sn > st[None, :]).sum(0) + 0.5 * (sn == st[None, :]).sum(0)
    return rank, float((1.0 / rank).mean()) if len(st) else 0.0


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
def forward_backward(state, graph, efeat, static, p, batch, k, n_heads, dt_source=0, loss_scale=1.0,
                     want_grads=True, relu_gates=None):
    """graph = event_list(src, dst, ts): neighbours by the scan of sample_recent (a build_adjacency tuple
    instead selects sample_recent_indexed).  batch = dict(src, dst, neg, eid, t).  Returns dict(loss,
    logits, grads, nbr, neid, nts, cnt, s_new, tau, z, ...).  Does not modify `state`.
    A batch with "labels" ([B, C]) is an edge-classification batch: no negative destinations, roots [src | dst],
    the head of edge_class_loss.
    relu_gates = (gate_z, gate_h), optional: see attention_bwd / decoder_bwd."""
    src, dst = (np.asarray(batch[n], np.int64) for n in ("src", "dst"))
    labels = batch.get("labels")
    # J sets of B negative destinations, one after the other (none in an edge-classification batch)
    neg = np.asarray(batch["neg"], np.int64).reshape(-1) if labels is None else np.zeros(0, np.int64)
    t = np.asarray(batch["t"], F)
    B = len(src); J = (len(neg) // B if B else 1) if labels is None else 0; R = (2 + J) * B
    d_m = state["mem"].shape[1]; d_t = p["time_w"].shape[0]
    root_node = np.concatenate([src, dst, neg]); root_t = np.concatenate([t] * (2 + J))
    if isinstance(graph, dict):
        nbr, neid, nts, cnt = sample_recent(graph["src"], graph["dst"], graph["ts"], root_node, root_t, k)
    else:
        nbr, neid, nts, cnt = sample_recent_indexed(graph, root_node, root_t, k)
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
    if labels is None:
        loss, logits, dc = decoder_loss(p, z[:B], z[B:2 * B], z[2 * B:])
    else:
        loss, logits, dc = edge_class_loss(p, z[:B], z[B:2 * B], labels)
    out = dict(loss=loss, logits=logits, nbr=nbr, neid=neid, nts=nts, cnt=cnt, s_new=s_new, tau=tau, z=z,
               dt_nbr=dt_nbr, zpre=ac["zpre"], hpre=dc["hpre"], gru_x=gc["x"], q_in=ac["q_in"], c_in=ac["c_in"])
    if not want_grads:
        return out

    gate_z, gate_h = relu_gates if relu_gates is not None else (None, None)
    if labels is None:
        g, dzs, dzd, dzn = decoder_bwd(p, dc, logits, loss_scale, gate_h)
    else:
        g, dzs, dzd = edge_class_bwd(p, dc, logits, loss_scale, gate_h)
        dzn = np.zeros((0, dzs.shape[1]), F)
    ga, dx_root, dx_nbr = attention_bwd(p, ac, np.concatenate([dzs, dzd, dzn], 0), n_heads, gate_z)
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
    msin = time_encode_darg(gc["delta"], p["time_w"], p["time_b"])
    g["time_w"] = g["time_w"] + (dphi * msin * gc["delta"][:, None]).sum(0)
    g["time_b"] = g["time_b"] + (dphi * msin).sum(0)
    out["grads"] = {n: g[n] for n in PARAM_NAMES}
    if static is not None:
        # co-trained static memory (Sec. 3.1): the static row of a node is an input of every slot that refers to the
        # node, so its gradient is the sum over those slots of the gradient reaching the static columns of x
        g_static = np.zeros(static.shape, F)
        np.add.at(g_static, root_node, dx_root[:, d_m:])
        np.add.at(g_static, nbr[valid], dx_nbr[valid][:, d_m:])
        out["g_static"] = g_static
    out["abs_terms"] = ac["abs_terms"]
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


def adam_init(p):
    """Adam's state: first and second moments (zero) and the step count."""
    return dict(m={n: np.zeros_like(p[n]) for n in PARAM_NAMES}, v={n: np.zeros_like(p[n]) for n in PARAM_NAMES}, t=0)


def adam(p, grads, st, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step with bias correction on every tensor except the time-encoding frequencies and phases:
    m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  p -= lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)."""
    st["t"] += 1
    t = st["t"]
    for n in PARAM_NAMES:
        if n in FROZEN_IN_SGD:
            continue
        g = grads[n]
        st["m"][n] = beta1 * st["m"][n] + (1.0 - beta1) * g
        st["v"][n] = beta2 * st["v"][n] + (1.0 - beta2) * g * g
        mhat = st["m"][n] / (1.0 - beta1 ** t)
        vhat = st["v"][n] / (1.0 - beta2 ** t)
        p[n] -= lr * mhat / (np.sqrt(vhat) + eps)


def apply_step(states, p, batches, outs, lr=0.0, adam_state=None, adam_hyper=(0.9, 0.999, 1e-8), static=None,
               lr_static=0.0):
    """Second half of a step, from the per-batch results `outs` of forward_backward: gradients summed over the
    batches (memory parallelism, Sec. 3.2.3: one weight set), loss averaged, the write-backs, one optimiser update
    (plain SGD, or Adam when adam_state is given).  static + lr_static: the co-trained static memory table (Sec. 3.1)
    takes static -= lr_static * g_static (rows no slot referred to have zero gradient)."""
    grads = {n: sum(o["grads"][n] for o in outs) for n in PARAM_NAMES}
    loss = float(np.mean([o["loss"] for o in outs]))
    wins = [apply_writeback(states[i], batches[i], outs[i]) for i in range(len(batches))]
    res = dict(loss=loss, grads=grads, outs=outs, winners=wins,
               abs_terms={n: sum(o["abs_terms"][n] for o in outs) for n in outs[0]["abs_terms"]})
    if "g_static" in outs[0]:
        res["g_static"] = sum(o["g_static"] for o in outs)
    if lr:
        if adam_state is not None:
            adam(p, grads, adam_state, lr, *adam_hyper)
        else:
            sgd(p, grads, lr)
    if static is not None and lr_static:
        static -= (lr_static * res["g_static"]).astype(static.dtype)
    return res


def train_step(states, graph, efeat, static, p, batches, k, n_heads, lr=0.0, dt_source=0):
    """One step over len(batches) memory replicas that share one weight set: replica i advances states[i] on
    batches[i], everything computed from the pre-step state and weights."""
    outs = [forward_backward(states[i], graph, efeat, static, p, batches[i], k, n_heads, dt_source)
            for i in range(len(batches))]
    return apply_step(states, p, batches, outs, lr)
