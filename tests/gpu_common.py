"""Shared helpers of the GPU parity tests: build one problem from the seeded generators, set it up on
the device (through the C-ABI binding) and in the oracle, and compare."""
import numpy as np

import synth
from oracle import tgnn_oracle as O

FP32_EPS = 2.0 ** -24
TOL = 1e-4   # spec bound: relative error (against the tensor's largest magnitude), fp32 path vs fp64 oracle


def rel_err(a, b, floor=1e-30):
    """max |a - b| / max(max |b|, floor)."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if a.size == 0:
        return 0.0
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), floor))


from synth import batch_np, custom_problem, make_problem  # noqa: E402,F401  (re-exported for the tests)

SCAN_LIMIT = 200_000   # event lists up to this length are scanned per query (the oracle's definition of the sampler);
                       # longer ones go through its indexed form, and spot_check_sampler scans for sampled roots


class OracleSide:
    def __init__(self, P, n_replicas=1, dt_source=0):
        d = P["d"]
        self.P, self.d, self.dt_source = P, d, dt_source
        self.scan = P["E"] <= SCAN_LIMIT
        self.adj = (O.event_list(P["src"], P["dst"], P["ts"]) if self.scan
                    else O.build_adjacency(P["src"], P["dst"], P["ts"], d.n_nodes))
        self.states = [O.new_state(d.n_nodes, d.d_mem) for _ in range(n_replicas)]
        self.p = O.to_f64(P["params"])
        self.static = P["static"]          # replaced by a float64 copy when the static memory is co-trained
        self.adam_state = None; self.adam_hyper = (0.9, 0.999, 1e-8); self.lr_static = 0.0

    def use_adam(self, beta1=0.9, beta2=0.999, eps=1e-8):
        self.adam_state = O.adam_init(self.p); self.adam_hyper = (beta1, beta2, eps)

    def train_static(self, lr_static):
        self.static = np.asarray(self.P["static"], np.float64).copy(); self.lr_static = lr_static

    def step(self, batches, replicas=None, lr=0.0, gpu=None):
        """One oracle step.  gpu (a GpuSide.step result of the same step, optional): where the GPU gated a ReLU
        pre-activation that lies within rounding of zero the other way (its fp32 value has the other sign), the
        oracle differentiates through the GPU's gate: that binary decision is taken once, in the kernel's
        precision, and the gradients of both sides are then those of the same function.  A gate that differs away
        from zero is an error.  The result carries the number of such ties as "relu_tie_flips"."""
        replicas = replicas if replicas is not None else list(range(len(batches)))
        sts = [self.states[r] for r in replicas]
        ef = self.P.get("efeat_host", self.P["efeat"])
        fb = lambda i, gates=None: O.forward_backward(sts[i], self.adj, ef, self.static, self.p, batches[i], self.d.k,
                                                      self.d.n_heads, self.dt_source, relu_gates=gates)
        outs = [fb(i) for i in range(len(batches))]
        flips = 0
        if gpu is not None:
            r0 = h0 = 0
            for i, o in enumerate(outs):
                nr, nh = o["zpre"].shape[0], o["hpre"].shape[0]
                gz = gpu["z"][r0:r0 + nr] > 0; gh = gpu["h1"][h0:h0 + nh] > 0
                r0 += nr; h0 += nh
                n_diff = 0
                for pre, gate in ((o["zpre"], gz), (o["hpre"], gh)):
                    diff = gate != (pre > 0)
                    assert np.all(np.abs(pre[diff]) <= 1e-5 * np.abs(pre).max()), "ReLU gate differs away from zero"
                    n_diff += int(diff.sum())
                if n_diff:
                    outs[i] = fb(i, (gz, gh))
                    flips += n_diff
            assert flips <= 8, flips
        res = O.apply_step(sts, self.p, batches, outs, lr, adam_state=self.adam_state, adam_hyper=self.adam_hyper,
                           static=self.static if self.lr_static else None, lr_static=self.lr_static)
        res["relu_tie_flips"] = flips
        return res


class GpuSide:
    def __init__(self, P, n_replicas=1, dt_source=0, own_stream=True, flags=0, max_neg_sets=1):
        """own_stream: run the steps on a stream of their own (the library then replays a captured HIP graph);
        False = the NULL stream, where every launch is enqueued directly."""
        import torch
        from paper_2307_07649_amd import tgnn
        self.torch, self.tgnn = torch, tgnn
        self.stream = torch.cuda.Stream() if own_stream else torch.cuda.default_stream()
        d = P["d"]
        self.P, self.d = P, d
        self.ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch,
                                n_replicas=n_replicas, dt_source=dt_source, flags=flags, max_neg_sets=max_neg_sets,
                                n_classes=d.n_classes)
        self.graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
        self.state = tgnn.State(d.n_nodes, d.d_mem, n_replicas, P["static"])
        self.params = tgnn.Params.from_numpy(P["params"])
        self.grads = tgnn.Params.zeros_like(self.params)
        self.loss = torch.zeros(4, device="cuda")

    def step(self, batches, replicas=None, lr=0.0, want=True, n_neg_sets=1):
        """want: True = every output; "gates" = only the two ReLU layers' outputs (what OracleSide.step(gpu=...) reads);
        False = nothing.  n_neg_sets > 1: every batch's "neg" holds that many sets, [J, n] (tgnn_train_step_epoch_parallel).
        Batches with "labels" ([n, C]): tgnn_train_step_edge_class (roots [src | dst], logits [sum n, C])."""
        torch, tgnn = self.torch, self.tgnn
        C = self.d.n_classes
        J = 0 if C else n_neg_sets
        replicas = replicas if replicas is not None else list(range(len(batches)))
        bl = [tgnn.Batch(b["src"], b["dst"], np.asarray(b["neg"]).reshape(-1), b["eid"], b["t"], replica=r)
              for b, r in zip(batches, replicas)]
        tot = sum(b.n for b in bl)
        n_logits = tot * C if C else (1 + J) * tot
        if not hasattr(self, "_out") or self._out[0].numel() != n_logits:      # stable output buffers: same graph key
            self._out = (torch.empty(n_logits, device="cuda"), torch.empty(2 * tot, dtype=torch.int32, device="cuda"))
        logits, win = self._out
        if C:
            labels = [torch.from_numpy(np.ascontiguousarray(b["labels"], np.float32)).cuda() for b in batches]
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            self.grads.zero_()
            if C:
                self.ctx.tgnn_train_step_edge_class(self.graph, self.state, self.params, self.grads, bl, labels, lr=lr,
                                                    out_loss=self.loss, out_logits=logits, out_winner=win)
            elif J == 1:
                self.ctx.tgnn_train_step(self.graph, self.state, self.params, self.grads, bl, lr=lr, out_loss=self.loss,
                                         out_logits=logits, out_winner=win)
            else:
                self.ctx.tgnn_train_step_epoch_parallel(self.graph, self.state, self.params, self.grads, bl, J, lr=lr,
                                                        out_loss=self.loss, out_logits=logits, out_winner=win)
        torch.cuda.synchronize()
        if not want:
            return None
        R = (2 + J) * tot; k = self.d.k
        if want == "gates":     # only what OracleSide.step needs to take the GPU's ReLU decisions
            dbg = self.ctx.tgnn_debug_read
            out = dict(z=dbg(6, torch.empty(R, self.d.d_mem, device="cuda")).cpu().numpy(),
                       h1=dbg(7, torch.empty(max(1 + J, 1) * tot, self.d.d_mem, device="cuda")).cpu().numpy())
            torch.cuda.synchronize()
            return out
        out = dict(loss=float(self.loss[0].item()), logits=logits.cpu().numpy().reshape((tot, C) if C else (-1,)),
                   winner=win.cpu().numpy(), grads=self.grads.numpy())
        dbg = self.ctx.tgnn_debug_read
        out["nbr"] = dbg(0, torch.empty(R, k, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["neid"] = dbg(1, torch.empty(R, k, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["nts"] = dbg(2, torch.empty(R, k, dtype=torch.float64, device="cuda")).cpu().numpy()
        out["cnt"] = dbg(3, torch.empty(R, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["s_new"] = dbg(4, torch.empty(R * (1 + k), self.d.d_mem, device="cuda")).cpu().numpy()
        out["tau"] = dbg(5, torch.empty(R * (1 + k), dtype=torch.float64, device="cuda")).cpu().numpy()
        out["z"] = dbg(6, torch.empty(R, self.d.d_mem, device="cuda")).cpu().numpy()
        out["h1"] = dbg(7, torch.empty(max(1 + J, 1) * tot, self.d.d_mem, device="cuda")).cpu().numpy()
        torch.cuda.synchronize()
        return out

    def eval_step(self, batches, n_neg_sets, replicas=None):
        """tgnn_eval_step: every batch's "neg" holds n_neg_sets sets, [J, n].  Returns logits [(1 + J) sum n], rank
        [sum n], the sum of the reciprocal ranks, winners, and the sampler's / UPDT's outputs like step()."""
        torch, tgnn = self.torch, self.tgnn
        J = n_neg_sets
        replicas = replicas if replicas is not None else list(range(len(batches)))
        bl = [tgnn.Batch(b["src"], b["dst"], np.asarray(b["neg"]).reshape(-1), b["eid"], b["t"], replica=r)
              for b, r in zip(batches, replicas)]
        tot = sum(b.n for b in bl)
        logits = torch.empty((1 + J) * tot, device="cuda"); win = torch.empty(2 * tot, dtype=torch.int32, device="cuda")
        rank = torch.empty(tot, device="cuda"); rr = torch.zeros(1, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            self.ctx.tgnn_eval_step(self.graph, self.state, self.params, bl, J, rank, rr, out_logits=logits, out_winner=win)
        torch.cuda.synchronize()
        R = (2 + J) * tot; k = self.d.k
        dbg = self.ctx.tgnn_debug_read
        out = dict(logits=logits.cpu().numpy(), rank=rank.cpu().numpy(), rr_sum=float(rr.item()), winner=win.cpu().numpy())
        out["nbr"] = dbg(0, torch.empty(R, k, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["cnt"] = dbg(3, torch.empty(R, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["z"] = dbg(6, torch.empty(R, self.d.d_mem, device="cuda")).cpu().numpy()
        torch.cuda.synchronize()
        return out

    def eval_class_step(self, batches, replicas=None):
        """tgnn_eval_step_edge_class on batches with "labels": logits [sum n, C], the (tp, fp, fn) counts of this call,
        winners."""
        torch, tgnn = self.torch, self.tgnn
        C = self.d.n_classes
        replicas = replicas if replicas is not None else list(range(len(batches)))
        bl = [tgnn.Batch(b["src"], b["dst"], np.asarray(b["neg"]).reshape(-1), b["eid"], b["t"], replica=r)
              for b, r in zip(batches, replicas)]
        tot = sum(b.n for b in bl)
        labels = [torch.from_numpy(np.ascontiguousarray(b["labels"], np.float32)).cuda() for b in batches]
        logits = torch.empty(tot * C, device="cuda"); win = torch.empty(2 * tot, dtype=torch.int32, device="cuda")
        counts = torch.zeros(3, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            self.ctx.tgnn_eval_step_edge_class(self.graph, self.state, self.params, bl, labels, counts, out_logits=logits,
                                               out_winner=win)
        torch.cuda.synchronize()
        return dict(logits=logits.cpu().numpy().reshape(tot, C), counts=tuple(int(x) for x in counts.cpu().numpy()),
                    winner=win.cpu().numpy())

    def state_np(self, replica=0):
        N = self.d.n_nodes
        s = slice(replica * N, (replica + 1) * N)
        st = self.state
        return dict(mem=st.mem[s].cpu().numpy(), mem_ts=st.mem_ts[s].cpu().numpy(), mail=st.mail[s].cpu().numpy(),
                    mail_ts=st.mail_ts[s].cpu().numpy(), mail_eid=st.mail_eid[s].cpu().numpy())


ERR_LOG = []    # (label, {quantity: measured relative error}) of every compared step, for the record


def compare_step(g, o_res, tol=TOL, check_grads=True, label=""):
    """g: GpuSide.step output (all batches concatenated); o_res: oracle step result.
    Indices and winners bit-exact.  Every floating-point tensor is held to `tol` relative to its OWN largest
    reference magnitude: logits, z, loss, s' of all R (1 + k) slots, and each of the 19 gradient tensors
    (|a - b| <= tol * max|b|).  For the four tensors fed only by the gradients of the attention scores (wq, bq, wk,
    bk) the bound is tol * max|b| + 16 eps_fp32 * A, with A the largest sum of the magnitudes of the tensor's
    summands before the cancellation in the softmax's backward pass (reported by the oracle): the softmax is invariant
    to a shift of a root's scores, so the exact gradient of bk is zero, and roots whose keys coincide contribute
    exact zeros to the other three; what both sides return there is rounding noise of summands of size A."""
    outs = o_res["outs"]
    # layout of the concatenated roots: per batch [src | dst | neg]
    nbr = np.concatenate([o["nbr"] for o in outs]); neid = np.concatenate([o["neid"] for o in outs])
    nts = np.concatenate([o["nts"] for o in outs]); cnt = np.concatenate([o["cnt"] for o in outs])
    assert np.array_equal(g["cnt"], cnt), label
    assert np.array_equal(g["nbr"], nbr), label
    assert np.array_equal(g["neid"], neid), label
    assert np.array_equal(g["nts"], nts), label
    assert np.array_equal(g["winner"], np.concatenate(o_res["winners"])), label
    logits = np.concatenate([o["logits"] for o in outs])
    errs = dict(logits=rel_err(g["logits"], logits), z=rel_err(g["z"], np.concatenate([o["z"] for o in outs])))
    R = len(cnt)
    n_roots = [len(o["cnt"]) for o in outs]
    s_all = np.concatenate([o["s_new"][:r] for o, r in zip(outs, n_roots)] + [o["s_new"][r:] for o, r in zip(outs, n_roots)])
    tau_all = np.concatenate([o["tau"][:r] for o, r in zip(outs, n_roots)] + [o["tau"][r:] for o, r in zip(outs, n_roots)])
    assert g["s_new"].shape == s_all.shape, label
    errs["s_new_all_slots"] = rel_err(g["s_new"], s_all)
    assert np.array_equal(g["tau"], tau_all), label                    # update times are copied, never computed
    errs["loss"] = abs(g["loss"] - o_res["loss"]) / max(abs(o_res["loss"]), 1e-30)
    # ReLU gates: a pre-activation within rounding of zero may be gated differently by the fp32 path and the fp64
    # oracle; OracleSide.step(gpu=g) has then differentiated through the GPU's gate (a gate that differs away from
    # zero fails there) and reports the number of such ties.
    assert "relu_tie_flips" in o_res, "compare_step needs an oracle step that was given the GPU's output (gpu=g)"
    flips = o_res["relu_tie_flips"]
    if check_grads:
        for n in O.PARAM_NAMES:
            ref = o_res["grads"][n]
            err = float(np.max(np.abs(g["grads"][n] - ref))) if ref.size else 0.0
            scale = float(np.max(np.abs(ref))) if ref.size else 0.0
            if n in o_res["abs_terms"]:
                # tensors fed only by the score gradients, which cancel inside the softmax's backward pass (exactly, for
                # bk and for identical keys): the bound adds 16 fp32 roundings of the largest sum of summand magnitudes
                floor = 16 * FP32_EPS * float(np.max(o_res["abs_terms"][n]))
                errs["g_" + n] = err / (scale + floor / tol) if scale + floor > 0 else 0.0
            elif scale == 0.0:       # e.g. the GRU tensors of a first batch: nothing consumed a mail
                assert not np.any(g["grads"][n]), (label, n, "gradient must be exactly zero")
                errs["g_" + n] = 0.0
            else:
                errs["g_" + n] = err / scale
    ERR_LOG.append((label, dict(errs, relu_tie_flips=float(flips))))
    bad = {k_: v for k_, v in errs.items() if not v <= tol}
    assert not bad, (label, "flips", flips, bad, errs)
    errs["relu_tie_flips"] = float(flips)
    return errs


def spot_check_sampler(P, g, batches, n=24, seed=0):
    """For graphs too long to scan for every root: the oracle's scan of the whole event list for n sampled roots of
    the step, against the neighbour rows the GPU returned (bit-exact)."""
    rng = np.random.default_rng(seed)
    roots = np.concatenate([np.concatenate([b["src"], b["dst"], b["neg"]]) for b in batches])
    times = np.concatenate([np.concatenate([b["t"], b["t"], b["t"]]) for b in batches])
    pick = rng.choice(len(roots), min(n, len(roots)), replace=False)
    k = P["d"].k
    nbr, ne, nts, cnt = O.sample_recent(P["src"], P["dst"], P["ts"], roots[pick], times[pick], k)
    assert np.array_equal(g["cnt"][pick], cnt) and np.array_equal(g["nbr"][pick], nbr)
    assert np.array_equal(g["neid"][pick], ne) and np.array_equal(g["nts"][pick], nts)


def dump_err_log(path):
    """Writes the measured errors of every compared step so far (one line per step) to `path`."""
    import json
    import os
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "a") as f:
        for label, e in ERR_LOG:
            f.write(json.dumps(dict(label=label, **{k_: float("%.3g" % v) for k_, v in e.items()})) + "\n")
    ERR_LOG.clear()


def compare_state(gs, ostate, tol=TOL, label=""):
    assert np.array_equal(gs["mail_eid"], ostate["mail_eid"].astype(np.int32)), label
    assert np.array_equal(gs["mail_ts"], ostate["mail_ts"]), label
    assert np.array_equal(gs["mem_ts"], ostate["mem_ts"]), label
    e1 = rel_err(gs["mem"], ostate["mem"]); e2 = rel_err(gs["mail"], ostate["mail"])
    assert e1 <= tol and e2 <= tol, (label, e1, e2)
    return e1, e2
