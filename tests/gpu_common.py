"""Shared helpers of the GPU parity tests: build one problem from the seeded generators, set it up on
the device (through the C-ABI binding) and in the oracle, and compare."""
import numpy as np

import synth
from oracle import tgnn_oracle as O

GRAD_TOL_TIE = 2e-3   # gradient bound on a step where a ReLU pre-activation tied at zero flipped (see compare_step)
TOL = 1e-4   # spec bound: relative error (against the tensor's largest magnitude), fp32 path vs fp64 oracle


def rel_err(a, b, floor=1e-30):
    """max |a - b| / max(max |b|, floor)."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if a.size == 0:
        return 0.0
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), floor))


def make_problem(name, n_events=None, random_phase=False, **dims_override):
    g = synth.gen_graph(name, n_events=n_events)
    d = synth.dims_of(name, **dims_override)
    E = len(g["src"])
    P = dict(name=name, d=d, src=g["src"], dst=g["dst"], ts=g["ts"], efeat=g["efeat"], E=E,
             neg=synth.gen_negatives(name, E), static=synth.gen_static(name),
             params=synth.gen_params(d, seed=synth.CONFIGS[name]["seed"], random_phase=random_phase))
    return P


def custom_problem(n_nodes, E, d_mem, d_time, d_edge, d_static, n_heads, k, batch, seed=0, tmax=100.0, ties=False):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n_nodes, E).astype(np.int32)
    dst = ((src + rng.integers(1, n_nodes, E)) % n_nodes).astype(np.int32)
    ts = np.sort(rng.integers(0, int(tmax), E).astype(np.float64)) if ties else np.sort(rng.uniform(0, tmax, E))
    d = synth.ModelDims(n_nodes=n_nodes, d_mem=d_mem, d_time=d_time, d_edge=d_edge, d_static=d_static,
                        n_heads=n_heads, k=k, batch=batch)
    return dict(name="custom", d=d, src=src, dst=dst, ts=ts, E=E,
                efeat=rng.standard_normal((E, d_edge)).astype(np.float32),
                neg=rng.integers(0, n_nodes, E).astype(np.int32),
                static=(0.1 * rng.standard_normal((n_nodes, d_static))).astype(np.float32) if d_static else None,
                params=synth.gen_params(d, seed=seed, random_phase=True))


def batch_np(P, lo, hi):
    return dict(src=P["src"][lo:hi], dst=P["dst"][lo:hi], neg=P["neg"][lo:hi],
                eid=np.arange(lo, hi, dtype=np.int32), t=P["ts"][lo:hi])


class OracleSide:
    def __init__(self, P, n_replicas=1, dt_source=0):
        d = P["d"]
        self.P, self.d, self.dt_source = P, d, dt_source
        self.adj = O.build_adjacency(P["src"], P["dst"], P["ts"], d.n_nodes)
        self.states = [O.new_state(d.n_nodes, d.d_mem) for _ in range(n_replicas)]
        self.p = O.to_f64(P["params"])

    def step(self, batches, replicas=None, lr=0.0):
        replicas = replicas if replicas is not None else list(range(len(batches)))
        sts = [self.states[r] for r in replicas]
        return O.train_step(sts, self.adj, self.P["efeat"], self.P["static"], self.p, batches, self.d.k,
                            self.d.n_heads, lr=lr, dt_source=self.dt_source)


class GpuSide:
    def __init__(self, P, n_replicas=1, dt_source=0, own_stream=True, flags=0):
        """own_stream: run the steps on a stream of their own (the library then replays a captured HIP graph);
        False = the NULL stream, where every launch is enqueued directly."""
        import torch
        from paper_2307_07649_amd import tgnn
        self.torch, self.tgnn = torch, tgnn
        self.stream = torch.cuda.Stream() if own_stream else torch.cuda.default_stream()
        d = P["d"]
        self.P, self.d = P, d
        self.ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch,
                                n_replicas=n_replicas, dt_source=dt_source, flags=flags)
        self.graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
        self.state = tgnn.State(d.n_nodes, d.d_mem, n_replicas, P["static"])
        self.params = tgnn.Params.from_numpy(P["params"])
        self.grads = tgnn.Params.zeros_like(self.params)
        self.loss = torch.zeros(4, device="cuda")

    def step(self, batches, replicas=None, lr=0.0, want=True):
        torch, tgnn = self.torch, self.tgnn
        replicas = replicas if replicas is not None else list(range(len(batches)))
        bl = [tgnn.Batch(b["src"], b["dst"], b["neg"], b["eid"], b["t"], replica=r) for b, r in zip(batches, replicas)]
        tot = sum(b.n for b in bl)
        if not hasattr(self, "_out") or self._out[0].numel() != 2 * tot:      # stable output buffers: same graph key
            self._out = (torch.empty(2 * tot, device="cuda"), torch.empty(2 * tot, dtype=torch.int32, device="cuda"))
        logits, win = self._out
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            self.grads.zero_()
            self.ctx.tgnn_train_step(self.graph, self.state, self.params, self.grads, bl, lr=lr, out_loss=self.loss,
                                     out_logits=logits, out_winner=win)
        torch.cuda.synchronize()
        if not want:
            return None
        R = 3 * tot; k = self.d.k
        out = dict(loss=float(self.loss[0].item()), logits=logits.cpu().numpy(), winner=win.cpu().numpy(),
                   grads=self.grads.numpy())
        dbg = self.ctx.tgnn_debug_read
        out["nbr"] = dbg(0, torch.empty(R, k, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["neid"] = dbg(1, torch.empty(R, k, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["nts"] = dbg(2, torch.empty(R, k, dtype=torch.float64, device="cuda")).cpu().numpy()
        out["cnt"] = dbg(3, torch.empty(R, dtype=torch.int32, device="cuda")).cpu().numpy()
        out["s_new"] = dbg(4, torch.empty(R * (1 + k), self.d.d_mem, device="cuda")).cpu().numpy()
        out["tau"] = dbg(5, torch.empty(R * (1 + k), dtype=torch.float64, device="cuda")).cpu().numpy()
        out["z"] = dbg(6, torch.empty(R, self.d.d_mem, device="cuda")).cpu().numpy()
        out["h1"] = dbg(7, torch.empty(2 * tot, self.d.d_mem, device="cuda")).cpu().numpy()
        torch.cuda.synchronize()
        return out

    def state_np(self, replica=0):
        N = self.d.n_nodes
        s = slice(replica * N, (replica + 1) * N)
        st = self.state
        return dict(mem=st.mem[s].cpu().numpy(), mem_ts=st.mem_ts[s].cpu().numpy(), mail=st.mail[s].cpu().numpy(),
                    mail_ts=st.mail_ts[s].cpu().numpy(), mail_eid=st.mail_eid[s].cpu().numpy())


def compare_step(g, o_res, tol=TOL, check_grads=True, label=""):
    """g: GpuSide.step output (all batches concatenated); o_res: oracle train_step result."""
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
    s_roots = np.concatenate([o["s_new"][:3 * len(o["logits"]) // 2] for o in outs])
    errs["s_new_roots"] = rel_err(g["s_new"][:R], s_roots)
    errs["loss"] = abs(g["loss"] - o_res["loss"]) / max(abs(o_res["loss"]), 1e-30)
    # ReLU gates: a pre-activation within rounding of zero may be gated differently by the fp32 path and the
    # fp64 oracle.  The outputs are continuous there (checked above at full tolerance) but the gradient is not,
    # so a step where such a tie flipped is compared at GRAD_TOL_TIE; any flip away from a tie is an error.
    zpre = np.concatenate([o["zpre"] for o in outs]); hpre = np.concatenate([o["hpre"] for o in outs])
    flips = 0
    for pre, act in ((zpre, g["z"]), (hpre, g["h1"])):
        diff = (act > 0) != (pre > 0)
        assert np.all(np.abs(pre[diff]) <= 1e-5 * np.abs(pre).max()), (label, "ReLU gate differs away from zero")
        flips += int(diff.sum())
    assert flips <= 4, (label, flips)
    errs["relu_tie_flips"] = 0.0
    if check_grads:
        gtol = tol if flips == 0 else GRAD_TOL_TIE
        # The key-bias gradient is identically zero in exact arithmetic (softmax is shift invariant), so a
        # tensor's error is taken relative to max(its own largest entry, 1e-3 of the largest gradient entry).
        gmax = max(float(np.max(np.abs(o_res["grads"][n]))) for n in O.PARAM_NAMES)
        for n in O.PARAM_NAMES:
            errs["g_" + n] = rel_err(g["grads"][n], o_res["grads"][n], floor=1e-3 * gmax)
    else:
        gtol = tol
    bad = {k_: v for k_, v in errs.items() if not (v <= (gtol if k_.startswith("g_") else tol))}
    assert not bad, (label, bad, errs)
    errs["relu_tie_flips"] = float(flips)
    return errs


def compare_state(gs, ostate, tol=TOL, label=""):
    assert np.array_equal(gs["mail_eid"], ostate["mail_eid"].astype(np.int32)), label
    assert np.array_equal(gs["mail_ts"], ostate["mail_ts"]), label
    assert np.array_equal(gs["mem_ts"], ostate["mem_ts"]), label
    e1 = rel_err(gs["mem"], ostate["mem"]); e2 = rel_err(gs["mail"], ostate["mail"])
    assert e1 <= tol and e2 <= tol, (label, e1, e2)
    return e1, e2
