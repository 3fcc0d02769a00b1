#!/usr/bin/env python3
"""Benchmark of the fused M-TGNN training step (tgnn_train_step) on one MI355X.

A step = one pass of the whole hot path over one mini-batch: sample -> gather -> time-encode -> GRU ->
attention -> decoder/BCE forward and backward -> SGD -> last-event-wins write-back.  Inputs (graph, edge
features, node state, weights, every mini-batch of the epoch) are resident in HBM before the clock starts.
Prints one JSON line; see the design doc for the roofline and cpu_baseline fields.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3

# HBM bytes per launch (read + written) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/train_step_C1_hbm_traffic.md (counter units scaled by the copy-kernel calibration described there).
# Counters cannot be read from inside this script, so the figures are the recorded ones, for C1 only.
MEASURED_TRAFFIC_BYTES = {"C1": {"kv_projection": 41.0e6, "assemble_ce": 33.8e6}}

STAGE_NAMES = ["(unused)", "(unused)", "roots + sample + distinct-node rows + prologue (pack weights, clear), one launch",
               "gather + time-encode (GRU input) + slot-to-row map", "GRU input + hidden projections (MFMA, one launch)", "(unused)",
               "(unused)", "GRU gates + slot-sort scan + per-slot attention input {e | Phi} (gather), one launch", "K/V projection of the slots (MFMA)",
               "per-node projections K, V, q, merge (MFMA)", "softmax attention + slot-sort fill", "merge layer (MFMA; only when the root chain does not fit)",
               "root chain: merge layer, decoder + loss, their backward down to the attention output (MFMA, one launch)",
               "decoder backward (only when the root chain does not fit)", "attention backward (softmax)",
               "per-node gradient sums; node projections + GRU gates backward with the keys' time-encoding gradients (one launch)",
               "all weight gradients (grouped MFMA GEMM)", "time-encoding gradients of the mails (MFMA) + write-back scatter + SGD (one launch)",
               "empty event bracket", "(unused)"]
STAGE_ASSEMBLE, STAGE_KV, STAGE_WGRAD, STAGE_EMPTY = 7, 8, 16, 18


def flops_wgrad(d, n_roots, n_rows):
    """Useful flops of the grouped weight-gradient launch, G += D^T A per problem (2 M N K each; bias gradients
    are one more column): decoder hidden layer and merge layer over the roots, the {e | Phi} columns of W_k / W_v as
    two products over the roots (a column of q / dO meets the d_e + d_t columns of its own head's block of the
    per-root sums; the launch also runs the blocks of tiles that straddle a head boundary, which are not counted),
    the node columns of W_k, W_v, W_q, W_o and the two GRU matrices over the distinct node rows."""
    R, U, dO = n_roots, n_rows, d.d_out
    macs = (R * 2 * dO * (dO + 1) + R * dO * dO + 2 * R * dO * (d.d_edge + d.d_time)
            + 2 * U * 2 * dO * (d.d_x + 1) + U * 3 * d.d_mem * (d.d_in + 1) + U * 3 * d.d_mem * (d.d_mem + 1))
    return 2.0 * macs


def flops_kv(d, n_roots):
    """Executed flops of the per-slot K/V projection: [R k, d_e + d_t] x [d_e + d_t, 2 d_o].  (The node part of
    the projection, d_x columns, is taken once per distinct node by another, much smaller GEMM.)"""
    return 2.0 * n_roots * d.k * (d.d_edge + d.d_time) * 2 * d.d_out


def assemble_bytes(d, n_roots):
    """Per-slot attention input: per neighbour slot read the edge-feature row, its index and the neighbour's
    update time, and write the {e | Phi} row and the time difference."""
    per_nbr = 4 * d.d_edge + 4 * (d.d_edge + d.d_time) + 4 + 8 + 8
    return n_roots * d.k * per_nbr


def gates_bytes(d, n_rows):
    """GRU gates, passenger of the same launch: per distinct node row read the two projections (6 d_m floats) and
    the stored memory, write the four gate values, the node row {s' | static} and clear the row's gradient
    accumulator (pitch 2 * pad32(2 d_o) floats)."""
    pad32 = lambda x: (x + 31) // 32 * 32
    return n_rows * 4 * (12 * d.d_mem + 2 * d.d_static + 2 * pad32(2 * d.d_out))


def step_flops(d, B):
    R = 3 * B; RK = R * d.k; S = R + RK
    gru = S * 2 * (d.d_in + d.d_mem) * 3 * d.d_mem
    attn = R * 2 * d.d_q * d.d_out + RK * 2 * 2 * d.d_kv * d.d_out + RK * 4 * d.d_out
    merge = R * 2 * (d.d_out + d.d_x) * d.d_out
    dec = 2 * B * (4 * d.d_out ** 2 + 2 * d.d_out)
    return 3.0 * (gru + attn + merge + dec)     # forward + backward ~ 3x forward


def step_bytes(d, B):
    R = 3 * B; RK = R * d.k; S = R + RK
    gather = S * (4 * d.d_mem + 8 * d.d_mem + 4 * d.d_edge + 4 * d.d_static + 20) + RK * 4 * d.d_edge
    sampler = R * (2 * d.k * 16 + 8 * 16)
    wb = 2 * B * (12 * d.d_mem + 20)
    return float(gather + sampler + wb)


def cpu_baseline(P, budget_s=15.0):
    """The oracle as it stands, timed on the host cores on the first mini-batches of the same workload."""
    from oracle import tgnn_oracle as O
    d = P["d"]
    adj = O.build_adjacency(P["src"], P["dst"], P["ts"], d.n_nodes)
    st = O.new_state(d.n_nodes, d.d_mem)
    p = O.to_f64(P["params"])
    ev = 0; steps = 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < budget_s and (steps + 1) * d.batch <= P["E"]:
        lo = steps * d.batch; hi = lo + d.batch
        b = dict(src=P["src"][lo:hi], dst=P["dst"][lo:hi], neg=P["neg"][lo:hi], eid=np.arange(lo, hi), t=P["ts"][lo:hi])
        O.train_step([st], adj, P["efeat"], P["static"], p, [b], d.k, d.n_heads, lr=1e-4)
        ev += hi - lo; steps += 1
    dt = time.perf_counter() - t0
    try:
        import threadpoolctl
        cores = max([i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return dict(value=ev / dt, unit="events/s", cores=int(cores), kind="oracle",
                sample=f"first {steps} mini-batches of {d.batch} events of {P['name']} from zero state "
                       f"(fp64 numpy, {dt:.1f} s)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=263)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C1", choices=["C0", "C1", "C2", "C3", "C4"])
    ap.add_argument("--events", type=int, default=None, help="shorten the event list (C4: default 2,000,000)")
    ap.add_argument("--lr", type=float, default=1e-4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--side-stream", action="store_true", help="let the library fork independent work of a step onto its second stream")
    ap.add_argument("--no-stage-events", action="store_true", help="do not time the two roofline kernels inside the timed region (every step then replays a captured HIP graph)")
    ap.add_argument("--steps-per-call", type=int, default=4,
                    help="consecutive training steps handed to the library per call (tgnn_train_steps; 1 = tgnn_train_step)")
    ap.add_argument("--event-every", type=int, default=16,
                    help="inside the timed region, every N-th step is launched kernel by kernel with HIP events around "
                         "the two roofline kernels; the other steps replay the captured HIP graph (1: every step)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run the library's plain copy kernel on 256 MiB three times (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2307_07649_amd import tgnn
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from gpu_common import make_problem

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    if args.calibrate_copy:
        a = torch.ones(64 << 20, device="cuda"); b = torch.empty_like(a)      # 256 MiB each
        for _ in range(3):
            tgnn.tgnn_debug_copy(b, a)
        torch.cuda.synchronize()
        del a, b

    name = args.config
    n_events = args.events
    if name == "C4" and n_events is None:
        n_events = 2_000_000
    P = make_problem(name, n_events=n_events)
    d = P["d"]
    nrep = d.n_replicas
    ctx = tgnn.Context(d.n_nodes, d.d_mem, d.d_time, d.d_edge, d.d_static, d.n_heads, d.k, d.batch, n_replicas=nrep,
                       flags=tgnn.FLAG_OVERWRITE_GRADS | (tgnn.FLAG_SIDE_STREAM if args.side_stream else 0))
    graph = tgnn.Graph(P["src"], P["dst"], P["ts"], d.n_nodes, P["efeat"])
    state = tgnn.State(d.n_nodes, d.d_mem, nrep, P["static"])
    params = tgnn.Params.from_numpy(P["params"])
    grads = tgnn.Params.zeros_like(params)
    loss = torch.zeros(4, device="cuda")
    loss_steps = torch.zeros(tgnn.MAX_STEPS_PER_CALL, device="cuda")

    # every mini-batch of the epoch, resident on the device
    import synth
    spans = synth.batches_of(P["E"], d.batch)
    M = len(spans)
    eid_all = np.arange(P["E"], dtype=np.int32)
    batches = [[tgnn.Batch(P["src"][lo:hi], P["dst"][lo:hi], P["neg"][lo:hi], eid_all[lo:hi], P["ts"][lo:hi], replica=r)
                for (lo, hi) in spans] for r in range(nrep)]
    shift = -(-M // nrep)

    def run_step(s):
        """Step s: replica r trains mini-batch (s + r*shift) mod M; a replica that wraps to mini-batch 0 starts a
        new epoch with its memory and mails reset."""
        bl = []
        for r in range(nrep):
            m = (s + r * shift) % M
            if m == 0 and s > 0:
                ctx.tgnn_state_reset(state, r)
            bl.append(batches[r][m])
        ctx.tgnn_train_step(graph, state, params, grads, bl, lr=args.lr, out_loss=loss)
        return sum(b.n for b in bl)

    per_call = max(1, min(args.steps_per_call, tgnn.MAX_STEPS_PER_CALL))
    last_loss = [(loss, 0)]   # where the most recent step's loss is

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
    torch.cuda.set_stream(torch.cuda.Stream())
    roof_mask = 0 if args.no_stage_events else (1 << STAGE_ASSEMBLE) | (1 << STAGE_KV) | (1 << STAGE_EMPTY)
    every = max(1, args.event_every)
    ctx.tgnn_profile_enable(roof_mask)
    ctx.tgnn_profile_every(2)             # warm up both launch modes
    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    ctx.tgnn_profile_enable(roof_mask)    # drops the warm-up's records
    ctx.tgnn_profile_every(every)
    ev = 0
    ev_timed_launches = 0                 # events of the steps whose roofline kernels were timed
    n_timed_launches = 0
    t0 = time.perf_counter()
    per_step = run_steps(args.warmup, args.warmup + args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert len(per_step) == args.steps
    ev = sum(per_step)
    if roof_mask != 0:
        timed = per_step[::every]             # the library times every `every`-th step, starting with the first
        ev_timed_launches, n_timed_launches = sum(timed), len(timed)
    final_loss = float(last_loss[0][0][last_loss[0][1]].item())
    n_g, ms_g = ctx.tgnn_profile_read(STAGE_ASSEMBLE)
    n_m, ms_m = ctx.tgnn_profile_read(STAGE_KV)
    n_e, ms_e = ctx.tgnn_profile_read(STAGE_EMPTY)
    ctx.tgnn_profile_enable(0)
    ctx.tgnn_profile_every(1)
    # A pair of HIP event records with nothing in between is itself several microseconds apart on this stack (the
    # step records such an empty bracket, stage 18, on the same steps).  It is reported, not subtracted: part of it
    # overlaps with a kernel's launch, so the difference would overstate the kernels.  The brackets are therefore
    # upper bounds of the launch durations (rocprofv3's kernel trace shows about 3 us less).
    bracket_us = ms_e / n_e * 1e3 if n_e else None
    kv_us = ms_m / n_m * 1e3 if n_m else None
    asm_us = ms_g / n_g * 1e3 if n_g else None

    # per-stage breakdown from a separate, untimed pass with every stage bracketed by events; the number of distinct
    # node rows of each of these steps is read back for the flops of the weight-gradient launch
    n_prof = min(args.steps, 64)
    ctx.tgnn_profile_enable((1 << len(STAGE_NAMES)) - 1)
    rows_step = torch.zeros(n_prof, dtype=torch.int32, device="cuda")
    ev_prof = 0
    for i, s in enumerate(range(args.warmup + args.steps, args.warmup + args.steps + n_prof)):
        ev_prof += run_step(s)
        ctx.tgnn_debug_read(8, rows_step[i:i + 1])
    torch.cuda.synchronize()
    stages = {}
    for i, nm in enumerate(STAGE_NAMES):
        c, ms = ctx.tgnn_profile_read(i)
        if c:
            stages[nm] = round(ms / c * 1e3, 2)
    n_w, ms_w = ctx.tgnn_profile_read(STAGE_WGRAD)
    n_e2, ms_e2 = ctx.tgnn_profile_read(STAGE_EMPTY)
    ctx.tgnn_profile_enable(0)
    rows_avg = float(rows_step.float().mean().item())
    wgrad_us = ms_w / n_w * 1e3 if n_w else None
    wgrad_tflops = flops_wgrad(d, 3 * ev_prof / n_prof, rows_avg) / (wgrad_us * 1e-6) / 1e12 if n_w else None

    ev_step = ev / args.steps
    R_avg = 3 * (ev_timed_launches / n_timed_launches if n_timed_launches else ev_step)   # roots per timed launch
    kv_tflops = flops_kv(d, R_avg) / (kv_us * 1e-6) / 1e12 if n_m else None
    asm_gbs = (assemble_bytes(d, R_avg) + gates_bytes(d, rows_avg)) / (asm_us * 1e-6) / 1e9 if n_g else None
    out = {
        "metric": "training events/sec (fwd+bwd+memory update) at 1 GPU",
        "value": ev / dt, "unit": "events/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: {d.n_nodes} nodes, {P['E']} events, d_mem {d.d_mem}, d_time {d.d_time}, "
                               f"d_edge {d.d_edge}, d_static {d.d_static}, {d.n_heads} heads, k {d.k}, "
                               f"batch {d.batch} x {nrep} replica(s), 1 negative/event, SGD lr {args.lr}",
                   "events_per_step": ev_step, "steps_per_call": per_call, "final_loss": final_loss},
        "roofline": {"bound": "mfma", "kernel": "gemm_nt_kernel: K/V projection of the {e | Phi} rows of all "
                                                "neighbour slots (fp32 MFMA 16x16x4), the longest forward kernel",
                     "achieved": kv_tflops, "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                     "frac": kv_tflops / PEAK_MFMA_F32_TFLOPS if kv_tflops else None,
                     "avg_launch_us": kv_us, "empty_event_bracket_us": bracket_us,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(name, {}).get("kv_projection")},
        "weight_gradients": {"bound": "mfma", "kernel": "gemm_tn_kernel: all weight gradients of the step in one grouped "
                                                        "launch (fp32 MFMA 16x16x4), the longest kernel of the step; timed "
                                                        "with HIP events in the untimed per-stage pass",
                             "achieved": wgrad_tflops, "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                             "frac": wgrad_tflops / PEAK_MFMA_F32_TFLOPS if wgrad_tflops else None,
                             "avg_launch_us": wgrad_us, "empty_event_bracket_us": ms_e2 / n_e2 * 1e3 if n_e2 else None,
                             "distinct_node_rows_per_step": rows_avg},
        "gather": {"bound": "hbm", "kernel": "assemble_ce_kernel: edge-feature row gather + time encoding into the "
                                             "per-slot key/value inputs; its first blocks carry the GRU gates of the "
                                             "distinct node rows (bytes of both counted)",
                   "achieved": asm_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                   "frac": asm_gbs / PEAK_HBM_GBS if asm_gbs else None,
                   "avg_launch_us": asm_us, "empty_event_bracket_us": bracket_us,
                   "traffic": MEASURED_TRAFFIC_BYTES.get(name, {}).get("assemble_ce")},
        "step_model": {"flops_per_step_per_slot_updt": step_flops(d, ev_step), "bytes_per_step": step_bytes(d, ev_step),
                       "note": "flops counted with UPDT per slot as the method states it; the library evaluates "
                               "UPDT once per distinct node, so executed flops are lower"},
        "stages_us": stages,
        "stages_us_note": "HIP-event brackets from an untimed pass launched kernel by kernel; every figure includes the "
                          "cost of an empty bracket (listed as its own entry)",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(P)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
