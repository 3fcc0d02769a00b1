#!/usr/bin/env python3
"""Benchmark of the fused M-TGNN training step (tgnn_train_step) on one MI355X.

A step = one pass of the whole hot path over one mini-batch: sample -> gather -> time-encode -> GRU ->
attention -> decoder/BCE forward and backward -> SGD -> last-event-wins write-back.  Inputs (graph, edge
features, node state, weights, every mini-batch of the epoch) are resident in HBM before the clock starts.

The headline (`value`) is the largest single-GPU configuration, C4: 16,682 nodes, the full 20,000,000-event list,
14.9 GB of edge features, mini-batches of 4,000 events.  The same run measures the other configurations (C0-C3 and C5, a graph without edge features)
(`configs`), and times the CPU oracle on the host cores (`cpu_baseline`).  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3

STAGE_NAMES = {2: "roots + sample + distinct-node rows + prologue (pack weights, clear), one launch",
               3: "state gather + time-encode (GRU input) + slot-to-row map",
               4: "GRU input + hidden projections (MFMA, one launch)",
               6: "GRU gates + slot-sort scan",
               9: "per-node projections K, V, q, merge (MFMA)",
               8: "per-node score vectors U = q W_k^c (MFMA)",
               10: "attention forward: edge-feature gather, time encoding, scores, softmax, weighted sums (+ slot-sort fill)",
               7: "attention output = node part + Zp W_v^c^T (MFMA)",
               11: "merge layer (MFMA; only when the root chain does not fit)",
               12: "root chain: merge layer, decoder + loss, their backward down to the attention output (MFMA, one launch)",
               13: "decoder backward (only when the root chain does not fit)",
               19: "G = dO W_v^c per root (MFMA)",
               14: "attention backward: edge-feature gather, time encoding, softmax backward, per-root sums",
               5: "dq = node part + Zs W_k^c^T (MFMA)",
               15: "per-node gradient sums; node projections + GRU gates backward",
               16: "all weight gradients + time-encoding gradients of the keys (grouped MFMA GEMM)",
               17: "time-encoding gradients of the mails (MFMA) + write-back scatter + SGD (one launch)",
               18: "empty event bracket"}
STAGE_GATHER, STAGE_ATTN_FWD, STAGE_ATTN_BWD, STAGE_WGRAD, STAGE_EMPTY = 3, 10, 14, 16, 18
N_STAGES = 20


# ---------------------------------------------------------------------------------------------------------
# work models: what the method asks for per slot, and what the library executes after its exact shortcuts
# ---------------------------------------------------------------------------------------------------------
def flops_per_slot_model(d, B):
    """The method as stated: UPDT for every one of the 3B(1+k) slots, unsplit projections; fwd + bwd ~ 3x fwd."""
    R = 3 * B; RK = R * d.k; S = R + RK
    gru = S * 2 * (d.d_in + d.d_mem) * 3 * d.d_mem
    attn = R * 2 * d.d_q * d.d_out + RK * 2 * 2 * d.d_kv * d.d_out + RK * 4 * d.d_out
    merge = R * 2 * (d.d_out + d.d_x) * d.d_out
    dec = 2 * B * (4 * d.d_out ** 2 + 2 * d.d_out)
    return 3.0 * (gru + attn + merge + dec)


def flops_wgrad(d, R, U):
    """Useful flops of the grouped weight-gradient launch, G += D^T A per problem (2 M N K each; a bias gradient is
    one more column): decoder hidden layer and merge layer over the roots, the {e | Phi} columns of W_k / W_v as two
    products over the roots (per-root sums against the query / output gradient of the same head), the node columns
    of W_k, W_v, W_q, W_o and the two GRU matrices over the distinct node rows."""
    dO = d.d_out
    macs = (R * 2 * dO * (dO + 1) + R * dO * dO + 2 * R * dO * (d.d_edge + d.d_time)
            + 2 * U * 2 * dO * (d.d_x + 1) + U * 3 * d.d_mem * (d.d_in + 1) + U * 3 * d.d_mem * (d.d_mem + 1))
    return 2.0 * macs


def flops_executed_model(d, B, U):
    """What the library's kernels execute for a step with U distinct (replica, node) rows among its slots: UPDT and
    the node part of every projection once per distinct row; the slots' own inputs {e | Phi} only meet per-root
    vectors (two dot products and two weighted sums of width H (d_e + d_t) per slot and direction); four products of
    width H (d_e + d_t) per root or node row tie those vectors to the weights; everything else per root.  Forward and
    backward listed separately (no 3x rule).  The products over H dcp columns are counted dense (as executed: the
    block-diagonal weights carry their zero blocks)."""
    R = 3 * B; RK = R * d.k; dO = d.d_out; dc = d.d_edge + d.d_time; Hdc = d.n_heads * dc
    fwd = (U * 2 * (d.d_in + d.d_mem) * 3 * d.d_mem          # GRU projections
           + U * 2 * d.d_x * 4 * dO                          # node part of K, V, q, merge
           + U * 2 * dO * Hdc                                # U = q W_k^c
           + RK * (2 * Hdc + 2 * dO) * 2                     # scores (u . c, q . Pk) and weighted sums (Zp, node part)
           + R * 2 * Hdc * dO                                # attention output from Zp
           + R * 2 * dO * dO + R * 2 * dO * 2 * dO           # merge (attention-output columns), decoder hidden layer
           + 2 * B * 2 * dO)                                 # logits
    bwd_data = (R * 2 * 2 * dO * dO + R * 2 * dO * dO        # dz, d(attention output)
                + R * 2 * dO * Hdc                           # G = dO W_v^c
                + RK * (2 * Hdc + 2 * dO) * 2                # dp (g . c, dO . Pv) and the sums Zs, dq (node part)
                + RK * 4 * d.n_heads * d.d_time              # gradient reaching the keys' time encoding
                + RK * 4 * dO                                # gradients of the neighbour rows' K and V, formed where summed
                + R * 2 * Hdc * dO                           # dq from Zs
                + U * 2 * 4 * dO * d.d_mem                   # node projections backward
                + U * 2 * 3 * d.d_mem * d.d_time)            # GRU input gradient onto the mails' time encoding
    return float(fwd + bwd_data + flops_wgrad(d, R, U))


def bytes_per_slot_model(d, B):
    """Algorithmic bytes of a step with nothing deduplicated: state + mail + edge-feature rows for every slot, edge
    features of the neighbour slots, sampler lists, write-back rows."""
    R = 3 * B; RK = R * d.k; S = R + RK
    gather = S * (4 * d.d_mem + 8 * d.d_mem + 4 * d.d_edge + 4 * d.d_static + 20) + RK * 4 * d.d_edge
    sampler = R * (2 * d.k * 16 + 8 * 16)
    wb = 2 * B * (12 * d.d_mem + 20)
    return float(gather + sampler + wb)


def attn_fwd_bytes(d, R, slots):
    """Attention forward launch, algorithmic bytes: per valid neighbour slot the edge-feature row, its index, the node
    row index, the neighbour's update time and the node's K and V rows; per root its q and U rows in, its softmax
    weights, node part of the output, per-head sums Zp and time differences out."""
    Hdcp = d.n_heads * ((d.d_edge + d.d_time + 3) // 4 * 4)
    per_slot = 4 * d.d_edge + 4 + 4 + 8 + 8 * d.d_out
    per_root = 4 * d.d_out + 4 * Hdcp + 4 + (4 * d.n_heads * d.k + 4 * d.d_out + 4 * Hdcp + 8 * d.k)
    return slots * per_slot + R * per_root


def attn_edge_bytes(d, slots):
    """Of those, the bytes that are a true HBM gather: the edge-feature rows (the table does not fit any cache on
    the large configuration; the node rows and per-root rows were written by the launches just before)."""
    return slots * 4 * d.d_edge


def state_gather_bytes(d, U):
    """State gather launch (memory, mail, the mail's edge-feature row -> GRU input and hidden rows): per distinct node
    row read 4 d_m + 8 d_m + 4 d_e + 20 bytes of state and write the same rows plus the time encoding."""
    return U * (2 * (12 * d.d_mem + 4 * d.d_edge) + 4 * d.d_time + 28)


def writeback_bytes(d, n_written):
    """Write-back scatter: per written node read s'_self, s'_other and write mem (4 d_m), mail (8 d_m), two times and
    the event id."""
    return n_written * (8 * d.d_mem + 12 * d.d_mem + 20)


def recorded_traffic(name, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of this workload
    (profiles/train_step_<name>_hbm_traffic.md, a line `traffic <kernel> <bytes>`); None when there is none.
    Counters cannot be read from inside this script."""
    path = os.path.join(ROOT, "profiles", f"train_step_{name}_hbm_traffic.md")
    try:
        for line in open(path):
            m = re.match(r"\s*traffic\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == kernel:
                return float(m.group(2))
    except OSError:
        pass
    return None


# ---------------------------------------------------------------------------------------------------------
# the oracle on the host cores
# ---------------------------------------------------------------------------------------------------------
def cpu_baseline(P, budget_s, threads):
    """The oracle as it stands, on the first mini-batches of the workload from zero state.  Its event list is cut
    after the last timed mini-batch: later events cannot precede any query of these batches, and the oracle's
    sampler scans the list it is given once per root.  threads: BLAS threads (None = all)."""
    from oracle import tgnn_oracle as O
    import threadpoolctl
    d = P["d"]
    n_max = min(P["E"] // d.batch, 6)
    cut = n_max * d.batch
    graph = O.event_list(P["src"][:cut], P["dst"][:cut], P["ts"][:cut])
    efeat = P["efeat_host"][np.arange(cut)] if "efeat_host" in P else P["efeat"][:cut]
    st = O.new_state(d.n_nodes, d.d_mem)
    p = O.to_f64(P["params"])
    ev = 0; steps = 0
    with threadpoolctl.threadpool_limits(limits=threads):
        used = max([i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()] + [1])
        t0 = time.perf_counter()
        while steps < n_max and (steps == 0 or time.perf_counter() - t0 < budget_s):
            lo = steps * d.batch; hi = lo + d.batch
            b = dict(src=P["src"][lo:hi], dst=P["dst"][lo:hi], neg=P["neg"][lo:hi], eid=np.arange(lo, hi), t=P["ts"][lo:hi])
            O.train_step([st], graph, efeat, P["static"], p, [b], d.k, d.n_heads, lr=1e-4)
            ev += hi - lo; steps += 1
        dt = time.perf_counter() - t0
    return dict(value=ev / dt, unit="events/s", cores=int(used), kind="oracle",
                sample=f"first {steps} mini-batch(es) of {d.batch} events of {P['name']} from zero state "
                       f"(fp64 numpy, {dt:.1f} s, {used} BLAS thread(s))")


# ---------------------------------------------------------------------------------------------------------
# one configuration on the GPU
# ---------------------------------------------------------------------------------------------------------
def build_problem(name, n_events):
    import synth
    if name == "C4" and (n_events is None or n_events > 4_000_000):
        # the edge-feature table of the full event list (14.9 GB) is drawn on the GPU, in chunks
        from synth.device import HostRowView, device_normal_table
        P = synth.make_problem(name, n_events=n_events, with_efeat=False)
        P["efeat"] = device_normal_table(P["E"], P["d"].d_edge, seed=synth.CONFIGS[name]["seed"] + 1000)
        P["efeat_host"] = HostRowView(P["efeat"])
        P["efeat_where"] = "drawn on the GPU in 2^20-row chunks (seeded)"
    else:
        P = synth.make_problem(name, n_events=n_events)
        P["efeat_where"] = "drawn on the host (seeded)"
    return P


def run_config(tgnn, torch, P, args, detail):
    """Warm-up, `args.steps` timed steps (replica r trains mini-batch (s + r * ceil(M / nrep)) mod M; a replica that
    wraps to mini-batch 0 starts a new epoch with its memory and mails reset), then an untimed pass with every stage
    bracketed by HIP events.  Returns the figures of the configuration."""
    import synth
    name = P["name"]; d = P["d"]; nrep = d.n_replicas
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch, n_replicas=nrep,
                       flags=tgnn.FLAG_OVERWRITE_GRADS | (tgnn.FLAG_SIDE_STREAM if args.side_stream else 0))
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
    state = tgnn.State(d.n_nodes, d.d_mem, nrep, P["static"])
    params = tgnn.Params.from_numpy(P["params"])
    grads = tgnn.Params.zeros_like(params)
    loss = torch.zeros(4, device="cuda")
    loss_steps = torch.zeros(tgnn.MAX_STEPS_PER_CALL, device="cuda")

    # every mini-batch of the epoch, resident on the device: the event arrays are uploaded once and sliced
    spans = synth.batches_of(P["E"], d.batch)
    M = len(spans)
    dsrc, ddst, dneg = (torch.from_numpy(np.ascontiguousarray(P[n], np.int32)).cuda() for n in ("src", "dst", "neg"))
    deid = torch.arange(P["E"], dtype=torch.int32, device="cuda")
    dts = torch.from_numpy(np.ascontiguousarray(P["ts"], np.float64)).cuda()
    batches = [[tgnn.Batch(dsrc[lo:hi], ddst[lo:hi], dneg[lo:hi], deid[lo:hi], dts[lo:hi], replica=r) for (lo, hi) in spans]
               for r in range(nrep)]
    shift = -(-M // nrep)

    def run_step(s):
        bl = []
        for r in range(nrep):
            m = (s + r * shift) % M
            if m == 0 and s > 0:
                ctx.tgnn_state_reset(state, r)
            bl.append(batches[r][m])
        ctx.tgnn_train_step(graph, state, params, grads, bl, lr=args.lr, out_loss=loss)
        return sum(b.n for b in bl)

    per_call = max(1, min(args.steps_per_call, tgnn.MAX_STEPS_PER_CALL))
    last_loss = [(loss, 0)]

    def run_steps(s_lo, s_hi):
        """Steps s_lo .. s_hi - 1, per_call of them per library call; a step at which a replica starts a new
        epoch (memory reset) begins a group of its own.  Returns the events of every step."""
        done = []
        s = s_lo
        while s < s_hi:
            group = []
            while s < s_hi and len(group) < per_call:
                ms = [(s + r * shift) % M for r in range(nrep)]
                if s > 0 and 0 in ms:
                    if group:
                        break
                    for r in range(nrep):
                        if ms[r] == 0:
                            ctx.tgnn_state_reset(state, r)
                group.append([batches[r][ms[r]] for r in range(nrep)])
                s += 1
            if len(group) == 1:
                ctx.tgnn_train_step(graph, state, params, grads, group[0], lr=args.lr, out_loss=loss)
                last_loss[0] = (loss, 0)
            else:
                ctx.tgnn_train_steps(graph, state, params, grads, group, lr=args.lr, out_loss=loss_steps)
                last_loss[0] = (loss_steps, len(group) - 1)
            done += [sum(b.n for b in bl) for bl in group]
        return done

    # a stream of its own: the library replays a captured HIP graph there (the NULL stream cannot be captured)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        roof_mask = 0 if args.no_stage_events else ((1 << STAGE_ATTN_FWD) | (1 << STAGE_ATTN_BWD) | (1 << STAGE_WGRAD)
                                                    | (1 << STAGE_GATHER) | (1 << STAGE_EMPTY))
        every = max(1, args.event_every)
        ctx.tgnn_profile_enable(roof_mask)
        ctx.tgnn_profile_every(2)             # warm up both launch modes
        run_steps(0, args.warmup)
        torch.cuda.synchronize()
        ctx.tgnn_profile_enable(roof_mask)    # drops the warm-up's records
        ctx.tgnn_profile_every(every)
        t0 = time.perf_counter()
        per_step = run_steps(args.warmup, args.warmup + args.steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert len(per_step) == args.steps
        ev = sum(per_step)
        timed = per_step[::every] if roof_mask else []     # the library times every `every`-th step, from the first on
        final_loss = float(last_loss[0][0][last_loss[0][1]].item())
        live = {st: ctx.tgnn_profile_read(st) for st in (STAGE_GATHER, STAGE_ATTN_FWD, STAGE_ATTN_BWD, STAGE_WGRAD, STAGE_EMPTY)}
        ctx.tgnn_profile_enable(0)
        ctx.tgnn_profile_every(1)

        # per-stage breakdown from a separate, untimed pass with every stage bracketed by events; the number of
        # distinct node rows of each of these steps is read back for the executed-work model
        n_prof = min(args.steps, 32)
        ctx.tgnn_profile_enable((1 << N_STAGES) - 1)
        rows_step = torch.zeros(n_prof, dtype=torch.int32, device="cuda")
        cnt_buf = torch.zeros(3 * d.batch * nrep, dtype=torch.int32, device="cuda")
        ev_prof = 0
        slots_prof = 0.0
        for i, s in enumerate(range(args.warmup + args.steps, args.warmup + args.steps + n_prof)):
            n_ev = run_step(s)
            ev_prof += n_ev
            ctx.tgnn_debug_read(8, rows_step[i:i + 1])
            ctx.tgnn_debug_read(3, cnt_buf[:3 * n_ev])          # sampled neighbours per root
            slots_prof += float(cnt_buf[:3 * n_ev].sum().item())
        torch.cuda.synchronize()
        stages = {}
        for i, nm in STAGE_NAMES.items():
            c, ms = ctx.tgnn_profile_read(i)
            if c:
                stages[nm] = round(ms / c * 1e3, 2)
        ctx.tgnn_profile_enable(0)
    rows_avg = float(rows_step.float().mean().item())

    def us(stage):
        n, ms = live[stage]
        return ms / n * 1e3 if n else None

    ev_step = ev / args.steps
    R_timed = 3 * (sum(timed) / len(timed) if timed else ev_step)      # roots per event-bracketed launch
    slots_per_root = slots_prof / (3 * ev_prof)                        # valid neighbour slots per root (measured)
    af_us, ab_us, wg_us, ga_us, empty_us = (us(s) for s in (STAGE_ATTN_FWD, STAGE_ATTN_BWD, STAGE_WGRAD, STAGE_GATHER, STAGE_EMPTY))
    wg_tf = flops_wgrad(d, R_timed, rows_avg) / (wg_us * 1e-6) / 1e12 if wg_us else None
    af_bytes = attn_fwd_bytes(d, R_timed, R_timed * slots_per_root)
    af_gbs = af_bytes / (af_us * 1e-6) / 1e9 if af_us else None
    ga_gbs = state_gather_bytes(d, rows_avg) / (ga_us * 1e-6) / 1e9 if ga_us else None
    ms_step = dt / args.steps * 1e3
    f_slot = flops_per_slot_model(d, ev_step); f_exec = flops_executed_model(d, ev_step, rows_avg)
    b_slot = bytes_per_slot_model(d, ev_step)
    res = {
        "workload": f"{name}: {d.n_nodes} nodes, {P['E']} events, d_mem {d.d_mem}, d_time {d.d_time}, d_edge {d.d_edge}, "
                    f"d_static {d.d_static}, {d.n_heads} heads, k {d.k}, batch {d.batch} x {nrep} replica(s), "
                    f"1 negative/event, SGD lr {args.lr}; edge features {P['efeat_where']}",
        "events_per_s": ev / dt, "ms_per_step": ms_step, "events_per_step": ev_step, "steps": args.steps,
        "final_loss": final_loss, "distinct_node_rows_per_step": rows_avg,
        "weight_gradients": {"tflops": wg_tf, "frac_of_mfma_peak": wg_tf / PEAK_MFMA_F32_TFLOPS if wg_tf else None,
                             "avg_launch_us": wg_us},
        "attention_fwd": {"gbs": af_gbs, "frac_of_hbm_peak": af_gbs / PEAK_HBM_GBS if af_gbs else None,
                          "avg_launch_us": af_us, "bytes_per_launch": af_bytes,
                          "edge_feature_bytes_per_launch": attn_edge_bytes(d, R_timed * slots_per_root),
                          "valid_slots_per_root": slots_per_root},
        "attention_bwd": {"avg_launch_us": ab_us},
        "state_gather": {"gbs": ga_gbs, "frac_of_hbm_peak": ga_gbs / PEAK_HBM_GBS if ga_gbs else None, "avg_launch_us": ga_us},
        "empty_event_bracket_us": empty_us,
        "step_model": {
            "flops_per_slot": f_slot, "flops_executed": f_exec, "bytes_per_slot": b_slot,
            "step_frac_of_mfma_peak_per_slot_count": f_slot / (ms_step * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS,
            "step_frac_of_mfma_peak_executed": f_exec / (ms_step * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS,
            "step_frac_of_hbm_peak_per_slot_bytes": b_slot / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "note": "per_slot: UPDT and unsplit projections for every slot, as the method states it (3 x forward); "
                    "executed: what the kernels run after the exact shortcuts (UPDT and node projections once per "
                    "distinct node; the slots' own inputs meet per-root vectors instead of being projected; weight "
                    "gradients of the slot projections over the roots); the per-slot count is never achieved work, a "
                    "fraction above 1 on it only says how much the shortcuts removed"},
    }
    if detail:
        res["stages_us"] = stages
        res["stages_us_note"] = ("HIP-event brackets from an untimed pass launched kernel by kernel; every figure includes "
                                 "the cost of an empty bracket (listed as its own entry)")
    # standalone write-back scatter (it rides inside the last launch of a step): 2 x batch occurrences per call
    n_ev = d.batch
    b0 = batches[0][min(M - 1, M // 2)]
    if b0.n == n_ev:
        s_src = torch.randn(n_ev, d.d_mem, device="cuda"); s_dst = torch.randn(n_ev, d.d_mem, device="cuda")
        tau = torch.zeros(n_ev, dtype=torch.float64, device="cuda")
        st2 = tgnn.State(d.n_nodes, d.d_mem, nrep, P["static"])
        n_wb = 50
        with torch.cuda.stream(stream):
            for _ in range(5):
                ctx.tgnn_memory_writeback(st2, 0, b0.src, b0.dst, b0.eid, b0.t, s_src, s_dst, tau, tau)
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(n_wb):
                ctx.tgnn_memory_writeback(st2, 0, b0.src, b0.dst, b0.eid, b0.t, s_src, s_dst, tau, tau)
            e1.record(stream)
            torch.cuda.synchronize()
        n_written = int(torch.unique(torch.cat([b0.src, b0.dst])).numel())
        call_us = e0.elapsed_time(e1) / n_wb * 1e3
        res["writeback_standalone"] = {
            "occurrences": 2 * n_ev, "nodes_written": n_written, "avg_call_us": call_us,
            "gbs": writeback_bytes(d, n_written) / (call_us * 1e-6) / 1e9,
            "note": "tgnn_memory_writeback alone: three small launches (descriptors, arbitration marks, scatter) per call, "
                    "timed back to back on one stream; bytes = rows read and written for the winners"}
    ctx.close()
    return res


def run_epoch_parallel(tgnn, torch, P, args, J):
    """tgnn_train_step_epoch_parallel on configuration P: J negative sets per positive mini-batch in one step (the
    one-GPU share of J epoch-parallel trainers).  Events/s counts positive events, as everywhere."""
    import synth
    d = P["d"]
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch, n_replicas=1,
                       flags=tgnn.FLAG_OVERWRITE_GRADS, max_neg_sets=J)
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
    state = tgnn.State(d.n_nodes, d.d_mem, 1, P["static"])
    params = tgnn.Params.from_numpy(P["params"]); grads = tgnn.Params.zeros_like(params)
    loss = torch.zeros(4, device="cuda")
    spans = [sp for sp in synth.batches_of(P["E"], d.batch) if sp[1] - sp[0] == d.batch]
    negs = np.stack([synth.gen_negatives(P["name"], P["E"], group=g) for g in range(J)])       # [J, E]
    dsrc, ddst = (torch.from_numpy(np.ascontiguousarray(P[n], np.int32)).cuda() for n in ("src", "dst"))
    deid = torch.arange(P["E"], dtype=torch.int32, device="cuda")
    dts = torch.from_numpy(np.ascontiguousarray(P["ts"], np.float64)).cuda()
    n_steps = min(args.steps, len(spans) - args.warmup)
    batches = [tgnn.Batch(dsrc[lo:hi], ddst[lo:hi], torch.from_numpy(np.ascontiguousarray(negs[:, lo:hi]).reshape(-1)).cuda(),
                          deid[lo:hi], dts[lo:hi]) for (lo, hi) in spans[:args.warmup + n_steps]]
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for b in batches[:args.warmup]:
            ctx.tgnn_train_step_epoch_parallel(graph, state, params, grads, [b], J, lr=args.lr, out_loss=loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b in batches[args.warmup:]:
            ctx.tgnn_train_step_epoch_parallel(graph, state, params, grads, [b], J, lr=args.lr, out_loss=loss)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    res = {"workload": f"{P['name']} with {J} negative sets per mini-batch (roots per step: {(2 + J) * d.batch})",
           "n_neg_sets": J, "steps": n_steps, "ms_per_step": dt / n_steps * 1e3,
           "positive_events_per_s": n_steps * d.batch / dt, "trained_pairs_per_s": n_steps * d.batch * (1 + J) / dt,
           "final_loss": float(loss[0].item())}
    ctx.close()
    return res


def run_edge_class(tgnn, torch, args, n_events=2_000_000, n_classes=56, n_true=6, d_edge=130):
    """tgnn_train_step_edge_class on the C4 graph recipe set up as the paper's own task on that graph (Sec. 4
    "Datasets"): 130 edge features, a 56-class head with 6 true classes per event, no negative destinations (roots
    [src | dst]).  First n_events events of the recipe; edge features and class targets are drawn on the GPU (seeded)."""
    import synth
    from synth.device import device_normal_table
    P = synth.make_problem("C4", n_events=n_events, with_efeat=False, with_labels=False, d_edge=d_edge, n_classes=n_classes)
    d = P["d"]
    efeat = device_normal_table(P["E"], d.d_edge, seed=synth.CONFIGS["C4"]["seed"] + 1000)
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch, n_replicas=1,
                       flags=tgnn.FLAG_OVERWRITE_GRADS, n_classes=n_classes)
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, efeat)
    state = tgnn.State(d.n_nodes, d.d_mem, 1, P["static"])
    params = tgnn.Params.from_numpy(P["params"]); grads = tgnn.Params.zeros_like(params)
    loss = torch.zeros(4, device="cuda")
    spans = [sp for sp in synth.batches_of(P["E"], d.batch) if sp[1] - sp[0] == d.batch]
    n_steps = min(args.steps, len(spans) - args.warmup)
    n_used = (args.warmup + n_steps) * d.batch
    gen = torch.Generator(device="cuda"); gen.manual_seed(synth.CONFIGS["C4"]["seed"] + 5000)
    # n_true distinct classes per event with a skewed class popularity (largest of exponential races)
    keys = torch.log(1.0 / (1.0 + torch.arange(n_classes, device="cuda", dtype=torch.float32)))[None, :] \
        - torch.log(-torch.log(torch.rand(n_used, n_classes, generator=gen, device="cuda").clamp_min(1e-12)))
    labels = torch.zeros(n_used, n_classes, device="cuda")
    labels.scatter_(1, keys.topk(n_true, dim=1).indices, 1.0)
    del keys
    dsrc, ddst = (torch.from_numpy(np.ascontiguousarray(P[n], np.int32)).cuda() for n in ("src", "dst"))
    deid = torch.arange(P["E"], dtype=torch.int32, device="cuda")
    dts = torch.from_numpy(np.ascontiguousarray(P["ts"], np.float64)).cuda()
    batches = [tgnn.Batch(dsrc[lo:hi], ddst[lo:hi], ddst[lo:hi], deid[lo:hi], dts[lo:hi])      # (neg is not read)
               for (lo, hi) in spans[:args.warmup + n_steps]]
    ys = [labels[lo:hi] for (lo, hi) in spans[:args.warmup + n_steps]]
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for b, y in zip(batches[:args.warmup], ys):
            ctx.tgnn_train_step_edge_class(graph, state, params, grads, [b], [y], lr=args.lr, out_loss=loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b, y in zip(batches[args.warmup:], ys[args.warmup:]):
            ctx.tgnn_train_step_edge_class(graph, state, params, grads, [b], [y], lr=args.lr, out_loss=loss)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    res = {"workload": f"C4 graph recipe, first {P['E']} events, d_edge {d.d_edge}, {n_classes}-class head with {n_true} true "
                       f"classes per event, batch {d.batch}, roots per step {2 * d.batch}, SGD lr {args.lr}",
           "steps": n_steps, "ms_per_step": dt / n_steps * 1e3, "events_per_s": n_steps * d.batch / dt,
           "final_loss": float(loss[0].item())}
    ctx.close()
    return res


def run_evaluation(tgnn, torch, P, args, J=49):
    """tgnn_eval_step on configuration P: the forward half with J sampled negative destinations per event, the rank of
    the true destination among them, the memory write-back (Sec. 4: 49 negatives, mean reciprocal rank)."""
    import synth
    d = P["d"]
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch, n_replicas=1,
                       max_neg_sets=J)
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
    state = tgnn.State(d.n_nodes, d.d_mem, 1, P["static"])
    params = tgnn.Params.from_numpy(P["params"])
    spans = [sp for sp in synth.batches_of(P["E"], d.batch) if sp[1] - sp[0] == d.batch]
    n_steps = min(args.steps, len(spans) - args.warmup)
    negs = np.stack([synth.gen_negatives(P["name"], P["E"], group=g) for g in range(J)])       # [J, E]
    dsrc, ddst = (torch.from_numpy(np.ascontiguousarray(P[n], np.int32)).cuda() for n in ("src", "dst"))
    deid = torch.arange(P["E"], dtype=torch.int32, device="cuda")
    dts = torch.from_numpy(np.ascontiguousarray(P["ts"], np.float64)).cuda()
    batches = [tgnn.Batch(dsrc[lo:hi], ddst[lo:hi], torch.from_numpy(np.ascontiguousarray(negs[:, lo:hi]).reshape(-1)).cuda(),
                          deid[lo:hi], dts[lo:hi]) for (lo, hi) in spans[:args.warmup + n_steps]]
    rank = torch.empty(d.batch, device="cuda"); rr = torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for b in batches[:args.warmup]:
            ctx.tgnn_eval_step(graph, state, params, [b], J, rank, rr)
        torch.cuda.synchronize()
        rr.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b in batches[args.warmup:]:
            ctx.tgnn_eval_step(graph, state, params, [b], J, rank, rr)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    res = {"workload": f"{P['name']}, {J} sampled negative destinations per event (roots per step: {(2 + J) * d.batch}), "
                       "forward half + ranks + memory write-back, untrained weights",
           "n_neg": J, "steps": n_steps, "ms_per_step": dt / n_steps * 1e3, "events_per_s": n_steps * d.batch / dt,
           "scored_pairs_per_s": n_steps * d.batch * (1 + J) / dt, "mean_reciprocal_rank": float(rr.item()) / (n_steps * d.batch)}
    ctx.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="all", choices=["all", "C0", "C1", "C2", "C3", "C4", "C5"],
                    help="all (default): the headline is C4 and the other configurations (C0-C3, C5) are measured in the same "
                         "run; Cn: only that configuration, which is then the headline")
    ap.add_argument("--events", type=int, default=None, help="shorten the event list of the headline configuration")
    ap.add_argument("--lr", type=float, default=1e-4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=10.0, help="seconds of oracle time per cpu_baseline leg")
    ap.add_argument("--side-stream", action="store_true", help="let the library fork independent work of a step onto its second stream")
    ap.add_argument("--no-stage-events", action="store_true", help="do not time kernels inside the timed region (every step then replays a captured HIP graph)")
    ap.add_argument("--steps-per-call", type=int, default=4,
                    help="consecutive training steps handed to the library per call (tgnn_train_steps; 1 = tgnn_train_step)")
    ap.add_argument("--event-every", type=int, default=16,
                    help="inside the timed region, every N-th step is launched kernel by kernel with HIP events around "
                         "the roofline kernels; the other steps replay the captured HIP graph (1: every step)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run the library's plain copy kernel on 256 MiB three times (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2307_07649_amd import tgnn

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    if args.calibrate_copy:
        a = torch.ones(64 << 20, device="cuda"); b = torch.empty_like(a)      # 256 MiB each
        for _ in range(3):
            tgnn.tgnn_debug_copy(b, a)
        torch.cuda.synchronize()
        del a, b

    head = "C4" if args.config == "all" else args.config
    others = [c for c in ("C0", "C1", "C2", "C3", "C5") if args.config == "all"]
    configs = {}
    epoch_parallel = evaluation = edge_class = None
    for name in others:
        P = build_problem(name, None)
        configs[name] = run_config(tgnn, torch, P, args, detail=False)
        print(f"bench.py: {name} {configs[name]['events_per_s']:.0f} events/s", file=sys.stderr, flush=True)
        if name == "C1":
            evaluation = run_evaluation(tgnn, torch, P, args)
            print(f"bench.py: C1 evaluation {evaluation['events_per_s']:.0f} events/s", file=sys.stderr, flush=True)
            epoch_parallel = run_epoch_parallel(tgnn, torch, P, args, 4)
        del P
    if args.config == "all":
        edge_class = run_edge_class(tgnn, torch, args)
        print(f"bench.py: edge classification {edge_class['events_per_s']:.0f} events/s", file=sys.stderr, flush=True)
        torch.cuda.empty_cache()
    P = build_problem(head, args.events)
    print(f"bench.py: {head} inputs ready", file=sys.stderr, flush=True)
    res = run_config(tgnn, torch, P, args, detail=True)
    configs[head] = {k: v for k, v in res.items() if k not in ("stages_us", "stages_us_note")}

    d = P["d"]
    wg = res["weight_gradients"]
    dom = dict(kernel="gemm_tn_kernel: all weight gradients of the step in one grouped launch (fp32 MFMA 16x16x4), the "
                      "longest launch of the step; useful flops of its nine products", tag="gemm_tn")
    dk = wg
    out = {
        "metric": "training events/sec (fwd+bwd+memory update) at 1 GPU",
        "value": res["events_per_s"], "unit": "events/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": res["workload"], "events_per_step": res["events_per_step"],
                   "steps_per_call": args.steps_per_call, "final_loss": res["final_loss"]},
        "roofline": {"bound": "mfma", "kernel": dom["kernel"], "achieved": dk["tflops"], "peak": PEAK_MFMA_F32_TFLOPS,
                     "unit": "TFLOP/s", "frac": dk["frac_of_mfma_peak"], "avg_launch_us": dk["avg_launch_us"],
                     "empty_event_bracket_us": res["empty_event_bracket_us"],
                     "traffic": recorded_traffic(head, dom["tag"])},
        "gather": {"bound": "hbm", "kernel": "fattn_fwd_fast_kernel: per root, gathers the edge-feature rows and node rows of its "
                                             "k neighbour slots, forms the time encoding, scores, softmax and weighted sums "
                                             "in registers",
                   "achieved": res["attention_fwd"]["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                   "frac": res["attention_fwd"]["frac_of_hbm_peak"],
                   "avg_launch_us": res["attention_fwd"]["avg_launch_us"],
                   "traffic": recorded_traffic(head, "fattn_fwd")},
        "state_gather": dict(res["state_gather"], bound="hbm", peak=PEAK_HBM_GBS,
                             kernel="gather_kernel: memory, mail and the mail's edge-feature row of every distinct node "
                                    "into the GRU input"),
        "writeback": res.get("writeback_standalone"),
        "weight_gradients": wg,
        "step_model": res["step_model"],
        "configs": configs,
        "epoch_parallel": epoch_parallel,
        "evaluation": evaluation,
        "edge_classification": edge_class,
        "stages_us": res.get("stages_us"), "stages_us_note": res.get("stages_us_note"),
    }
    if not args.no_cpu_baseline:
        allc = cpu_baseline(P, args.cpu_budget, None)
        one = cpu_baseline(P, args.cpu_budget, 1)
        out["cpu_baseline"] = dict(allc, single_thread=one, host_cores=os.cpu_count())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
