#!/usr/bin/env python3
"""Benchmark of the DSGD-CECA hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: one dsgd_ceca_step call
(gradient + CECA round fused) for the training workloads, one ceca_gossip_round call for the pure
gossip workloads.  Inputs are generated on the device before the timed region.  Prints ONE JSON line.

The default run also times every other configuration briefly (`configs`) and, before the process first
touches the GPU, the CPU oracle on one thread and on all host cores (`cpu_baseline`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--others] [--mix-only] [--no-cpu]
                    [--no-configs] [--eager-only] [--copy-probe] [--write-data FILE | --data-file FILE]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
EAGER_ONLY = False      # --eager-only: minibatch workloads skip the HIP-graph and multi-iteration legs
NO_GRAPH = False        # --no-graph: minibatch workloads skip only the HIP-graph leg (for hardware-counter passes)
DATA_FILE = None        # --data-file / --write-data: minibatch inputs handed over by file
WRITE_DATA = False
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import workloads as WL  # noqa: E402

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth

# Algorithmic HBM bytes per agent-parameter per call, fp32 state [x; y]: every distinct array element
# moved once.  (read, read in round 0 where b = 0 and y is not needed, written)
#   gossip round      x, y read (x only in round 0), x+, y+ written
#   fused quad step   x, y, c read (x, c in round 0), x+, y+ written
# The "gather model" figure also charges the peer row as a separate read, the way a plain row-gather
# kernel pays it (+4 for gossip, +8 for the fused step with its centre row); the one-port pair kernel
# and this build's chain walk do not pay it.
ALG_BYTES = {"gossip": (8.0, 4.0, 8.0), "quad_center": (12.0, 8.0, 8.0)}
GATHER_EXTRA = {("gossip", 1): 0.0, ("gossip", 2): 4.0, ("quad_center", 1): 0.0, ("quad_center", 2): 8.0}


def chain_bytes(kind: str, port: int, rounds):
    """Mean algorithmic and gather-model bytes per agent-parameter over the given round numbers."""
    rd, rd0, wr = ALG_BYTES[kind]
    alg = sum((rd0 if r == 0 else rd) + wr for r in rounds) / len(rounds)
    return alg, alg + GATHER_EXTRA[(kind, port)]


def minibatch_bytes(B: int):
    # A_B rows once, z once, x, y read, x+, y+ written | model: A_B twice, z twice, v written and read twice
    return 4.0 * B + 16.0, 8.0 * B + 36.0


def _tau(n):
    return (n - 1).bit_length()


def _ld(d):
    """Leading dimension of the stacked state: rows start on 256-byte boundaries."""
    return (d + 63) // 64 * 64


class Timer:
    """HIP events on the stream the kernels are launched on (torch's current stream) + host clock."""

    def __init__(self, torch):
        self.torch = torch
        self.e0 = torch.cuda.Event(enable_timing=True)
        self.e1 = torch.cuda.Event(enable_timing=True)

    def __enter__(self):
        self.torch.cuda.synchronize()
        self.t0 = time.perf_counter()
        self.e0.record()
        return self

    def __exit__(self, *a):
        self.e1.record()
        self.torch.cuda.synchronize()
        self.wall_ms = (time.perf_counter() - self.t0) * 1e3
        self.event_ms = self.e0.elapsed_time(self.e1)


def per_step_events(torch, step, ks):
    """Milliseconds of each step in `ks`, from HIP events recorded between the launches (a pass of its own,
    after the timed region: the events must not sit inside the figure that `value` is computed from)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(ks) + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for j, k in enumerate(ks):
        step(k)
        ev[j + 1].record()
    torch.cuda.synchronize()
    return [ev[j].elapsed_time(ev[j + 1]) for j in range(len(ks))]


def frac_distribution(ms_list, ks, tau, kind, units):
    """min / median / max over the steps of (algorithmic bytes of that step's round) / time / peak."""
    rd, rd0, wr = ALG_BYTES[kind]
    fr = sorted(units * ((rd0 if k % tau == 0 else rd) + wr) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS for ms, k in zip(ms_list, ks))
    r0 = [units * (rd0 + wr) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS for ms, k in zip(ms_list, ks) if k % tau == 0]
    out = {"min": fr[0], "median": fr[len(fr) // 2], "max": fr[-1], "steps": len(fr)}
    if r0:
        out["round0_median"] = sorted(r0)[len(r0) // 2]
    return out


def probe(torch, P, arrays, cnt, reads, writes, reps=10):
    """Milliseconds and GB/s of the elementwise probe kernel with this mix of streaming reads and writes."""
    a, b, c, o1, o2 = arrays
    for _ in range(3):
        P.ceca_stream_probe(a, b, c, o1, o2, cnt, reads=reads, writes=writes)
    with Timer(torch) as tp:
        for _ in range(reps):
            P.ceca_stream_probe(a, b, c, o1, o2, cnt, reads=reads, writes=writes)
    ms = tp.event_ms / reps
    return ms, 4.0 * (reads + writes) * cnt / (ms * 1e-3) / 1e9


def consensus_report(torch, P, X, n, d, ld):
    """Consensus observables of the x rows, measured by the library (outside any timed region)."""
    ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    P.consensus_error(X, n, d, out, workspace=ws, ld=ld)
    torch.cuda.synchronize()
    frob2, resid, mx, nrm, _ = out.tolist()
    return {"max_dev_over_mean_norm": mx / nrm if nrm else None, "mean_distance_to_average": resid / n,
            "mean_norm": nrm}


def run_quad(torch, P, Bn, sp, steps, warmup):
    n, d, port = sp.n, sp.d, sp.port
    ld = _ld(d)
    c = torch.empty((n, ld), dtype=torch.float32, device="cuda")
    WL.device_normal((n, ld), seed=sp.seed, out=c)
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
    T = S if port == 1 else torch.empty_like(S)
    tau = _tau(n)

    def step(k):
        nonlocal S, T
        P.dsgd_ceca_step(S, T, n, d, Bn.make_quad_center_loss(c, sp.noise_std, sp.seed, k), None, sp.lr,
                         k % tau, port, ld=ld)
        if port == 2:
            S, T = T, S

    for k in range(warmup):
        step(k)
    with Timer(torch) as tm:
        for k in range(warmup, warmup + steps):
            step(k)
    # the same steps once more with an event after each, for the spread of the per-step fraction of peak
    ks = list(range(warmup + steps, warmup + 2 * steps))
    tm.frac = frac_distribution(per_step_events(torch, step, ks), ks, tau, "quad_center", n * d)
    # what the device gives the simplest kernel with each round's traffic mix (same array sizes, no indexing):
    # 3 streaming reads + 2 streaming writes per element for a full round, 2 + 2 for round 0 (y is not read);
    # out of place, and in place (what the one-port rounds do)
    pa, pb = S[:n].reshape(-1), S[n:].reshape(-1)
    po1, po2 = (pa, pb) if port == 1 else (T[:n].reshape(-1), T[n:].reshape(-1))
    cnt = n * ld
    arrays = (pa, pb, c.reshape(-1), po1, po2)
    ms32, gb32 = probe(torch, P, arrays, cnt, 3, 2)
    # round 0 reads x and c: the probe's two reads are its first two arrays
    ms22, gb22 = probe(torch, P, (pa, c.reshape(-1), None, po1, po2), cnt, 2, 2)
    tm.probe = {"stream_probe_ms": ms32, "stream_probe_GBs": gb32,
                "stream_probe_round0_ms": ms22, "stream_probe_round0_GBs": gb22}
    if port == 2:
        msip, gbip = probe(torch, P, (pa, pb, c.reshape(-1), pa, pb), cnt, 3, 2)
        tm.probe.update({"stream_probe_in_place_ms": msip, "stream_probe_in_place_GBs": gbip})
    # the same step with gradients the caller supplies (any loss, e.g. from autograd): same traffic, no noise
    # arithmetic; c stands in for the gradient rows
    gl = Bn.make_gradient_loss(c)
    tc = Timer(torch)
    with tc:
        for k in range(2 * tau):
            P.dsgd_ceca_step(S, T, n, d, gl, None, sp.lr, k % tau, port, ld=ld)
            if port == 2:
                S, T = T, S
    tm.probe["caller_gradient_step_ms"] = tc.event_ms / (2 * tau)
    S.zero_()
    # the same iterations fused: up to 50 per dsgd_ceca_steps call (same bits as the calls above), 20 bytes
    # per agent-parameter per call; bound by the noise generator's arithmetic, not by HBM
    K = min(steps, 50)
    loss0 = Bn.make_quad_center_loss(c, sp.noise_std, sp.seed, warmup + steps)
    P.dsgd_ceca_steps(S, T, n, d, loss0, sp.lr, (warmup + steps) % tau, min(K, 5), port, ld=ld)
    with Timer(torch) as tf:
        P.dsgd_ceca_steps(S, T, n, d, loss0, sp.lr, (warmup + steps) % tau, K, port, ld=ld)
    tm.fused = {"fused_iterations_per_call": K, "fused_ms_per_iteration": tf.event_ms / K,
                "fused_agent_param_updates_per_s": n * d * K / (tf.event_ms * 1e-3)}
    return tm, 1, chain_bytes("quad_center", port, [k % tau for k in range(warmup, warmup + steps)])


def run_gossip(torch, P, Bn, sp, steps, warmup):
    n, d, port = sp.n, sp.d, sp.port
    ld = _ld(d)
    S = torch.empty((2 * n, ld), dtype=torch.float32, device="cuda")
    WL.device_normal((n, ld), seed=sp.seed, out=S[:n])
    S[n:] = S[:n]
    T = S if port == 1 else torch.empty_like(S)
    tau = _tau(n)

    def step(k):
        nonlocal S, T
        P.ceca_gossip_round(S, T, n, d, k % tau, port, ld=ld)
        if port == 2:
            S, T = T, S

    for k in range(warmup):
        step(k)
    with Timer(torch) as tm:
        for k in range(warmup, warmup + steps):
            step(k)
    ks = list(range(warmup + steps, warmup + 2 * steps))
    tm.frac = frac_distribution(per_step_events(torch, step, ks), ks, tau, "gossip", n * d)
    # the simplest kernel with a round's traffic mix: x, y read and written (x only read in round 0)
    pa, pb = S[:n].reshape(-1), S[n:].reshape(-1)
    po1, po2 = (pa, pb) if port == 1 else (T[:n].reshape(-1), T[n:].reshape(-1))
    ms22, gb22 = probe(torch, P, (pa, pb, None, po1, po2), n * ld, 2, 2)
    ms12, gb12 = probe(torch, P, (pa, None, None, po1, po2), n * ld, 1, 2)
    tm.probe = {"stream_probe_ms": ms22, "stream_probe_GBs": gb22, "stream_probe_round0_ms": ms12,
                "stream_probe_round0_GBs": gb12}
    # consensus error after each of the tau rounds from a fresh X(0) (not timed)
    WL.device_normal((n, ld), seed=sp.seed, out=S[:n])
    S[n:] = S[:n]
    per_round = []
    for r in range(tau):
        P.ceca_gossip_round(S, T, n, d, r, port, ld=ld)
        if port == 2:
            S, T = T, S
        per_round.append(consensus_report(torch, P, S[:n], n, d, ld)["max_dev_over_mean_norm"])
    tm.consensus = {"max_dev_over_mean_norm_after_round": per_round}
    # all tau rounds fused into one pass (exact averaging): 12 bytes per agent-parameter in total
    for _ in range(2):
        P.ceca_gossip_rounds(S, T, n, d, tau, port, ld=ld)
    reps = max(1, steps // tau)
    with Timer(torch) as tf:
        for _ in range(reps):
            P.ceca_gossip_rounds(S, T, n, d, tau, port, ld=ld)
    # all of them as exact averaging (x in, x out: 8 bytes), and the simplest kernels with those two mixes
    for _ in range(2):
        P.ceca_average(S[:n], T[:n], n, d, port, ld=ld)
    with Timer(torch) as ta:
        for _ in range(reps):
            P.ceca_average(S[:n], T[:n], n, d, port, ld=ld)
    ms11, gb11 = probe(torch, P, (pa, None, None, po1, None), n * ld, 1, 1)
    tm.fused = {"fused_rounds": tau, "fused_ms": tf.event_ms / reps, **tm.consensus,
                "fused_GBs_on_12B": n * d * 12.0 / (tf.event_ms / reps * 1e-3) / 1e9,
                "fused_probe_1r2w_ms": ms12,
                "average_ms": ta.event_ms / reps, "average_GBs_on_8B": n * d * 8.0 / (ta.event_ms / reps * 1e-3) / 1e9,
                "average_probe_1r1w_ms": ms11}
    return tm, 1, chain_bytes("gossip", port, [k % tau for k in range(warmup, warmup + steps)])


def run_minibatch(torch, P, Bn, sp, steps, warmup):
    n, d, port, N, B = sp.n, sp.d, sp.port, sp.N, sp.B
    if DATA_FILE and not WRITE_DATA:
        # inputs drawn by an earlier process (python bench.py --workload NAME --write-data FILE): this process
        # then issues no generator kernels before the library's own
        Ah = np.load(DATA_FILE + ".A.npy", mmap_mode="r")
        th = np.load(DATA_FILE + ".t.npy")
        assert Ah.shape == (n, N, d) and th.shape == (n, N), "data file does not match the workload"
        A = torch.empty((n, N, d), dtype=torch.float32, device="cuda")
        for i0 in range(0, n, 64):                       # in slices: the host copy is memory-mapped
            A[i0:i0 + 64].copy_(torch.from_numpy(np.ascontiguousarray(Ah[i0:i0 + 64])))
        t = torch.from_numpy(th).cuda()
    elif sp.name.startswith("logistic1023"):
        A, t, _ = WL.device_logistic_sparse(n, N, d, sp.seed)
    else:
        if sp.loss == "lsq":
            Ah, th, _ = WL.lsq_data(n, N, d, sp.seed, obs_noise=sp.obs_noise)
        else:
            Ah, th, _ = WL.logistic_data_hetero(n, N, d, sp.seed)
        A, t = torch.from_numpy(Ah).cuda(), torch.from_numpy(th).cuda()
    if WRITE_DATA:
        np.save(DATA_FILE + ".A.npy", A.cpu().numpy())
        np.save(DATA_FILE + ".t.npy", t.cpu().numpy())
        print(f"bench.py: wrote {DATA_FILE}.A.npy and .t.npy", file=sys.stderr)
        sys.exit(0)
    if sp.B == sp.N:
        idx_h = WL.full_batch_indices(n, N)
    else:
        idx_h = WL.batch_indices(n, N, B, min(steps + warmup, 256), sp.seed)
    nidx = idx_h.shape[0]
    idx = torch.from_numpy(idx_h).cuda()
    kind = Bn.LOSS_LSQ if sp.loss == "lsq" else Bn.LOSS_LOGISTIC

    def make_loss(k):
        return Bn.make_minibatch_loss(kind, A, t, N, B, grad_scale=sp.grad_scale, noise_std=sp.noise_std,
                                      seed=sp.seed, k=k)

    loss0 = make_loss(0)
    ws = torch.empty(max(P.dsgd_ceca_workspace_bytes(n, d, loss0), 256), dtype=torch.uint8, device="cuda")
    ld = _ld(d)
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
    T = S if port == 1 else torch.empty_like(S)
    tau = _tau(n)

    def step(k):
        nonlocal S, T
        loss = make_loss(k) if sp.noise_std else loss0
        P.dsgd_ceca_step(S, T, n, d, loss, idx[k % nidx], WL.step_size(sp, k), k % tau, port, workspace=ws, ld=ld)
        if port == 2:
            S, T = T, S

    for k in range(warmup):
        step(k)
    with Timer(torch) as tm:
        for k in range(warmup, warmup + steps):
            step(k)
    tm.final = consensus_report(torch, P, S[:n], n, d, ld)      # after warmup + steps iterations from x(0) = 0
    one_kernel_gradient = (d % 4 == 0 and ((n >= 128 and 1024 < d <= 16384) or (B <= 32 and d <= 1024) or (B <= 16 and d <= 4096)
                                           or (B <= 8 and d <= 8192) or (B <= 4 and d <= 16384))) or (d % 4 != 0 and d <= 1024)
    launches = 2 if one_kernel_gradient else 3
    if EAGER_ONLY:
        return tm, launches, minibatch_bytes(B)
    # launch-bound loops: the same iterations captured once as a HIP graph and replayed
    window = 2 * tau * max(1, 16 // tau)          # even number of steps: two-port buffers end where they began
    if not NO_GRAPH:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for k in range(window):
                step(k)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for k in range(window):
                step(k)
        reps = max(1, steps // window)
        graph.replay()
        with Timer(torch) as tg:
            for _ in range(reps):
                graph.replay()
        tm.graph_ms_per_step = tg.event_ms / (reps * window)
    # the same iterations through dsgd_ceca_run (one call for a window of iterations; with many agents one
    # kernel per iteration): needs one step size and a batch table that covers the window
    # (a decaying step size is constant over windows of lr_decay_every iterations: one call per window)
    K = sp.lr_decay_every if sp.lr_decay_every else min(steps, nidx)
    idx_run = idx[:K] if nidx >= K else idx[:1].repeat(K, 1, 1).contiguous()     # a full batch serves every iteration
    if K >= 2:
        wsr = torch.empty(P.dsgd_ceca_run_workspace_bytes(n, d, loss0) + 256, dtype=torch.uint8, device="cuda")
        wsr = wsr[(-wsr.data_ptr()) % 256:]
        calls = max(1, steps // K)

        def run_windows():
            for w in range(calls):
                P.dsgd_ceca_run(S, T, n, d, make_loss(w * K) if sp.noise_std else loss0, idx_run, WL.step_size(sp, w * K),
                                (w * K) % tau, K, port, workspace=wsr, ld=ld)

        run_windows()
        with Timer(torch) as tr:
            run_windows()
        tm.run_ms_per_step = tr.event_ms / (calls * K)
        tm.run_iterations_per_call = K
    return tm, launches, minibatch_bytes(B)


def run_consensus(torch, P, Bn, steps=20, warmup=3):
    """consensus_error (x read once: 4 algorithmic bytes per agent-parameter) at the sizes of the three
    configurations that report it, on the row pitch the other legs use; the allocation-free entry point beside
    it; and the read-only probe on the same bytes."""
    out = []
    for name in ("quad31_2p", "gossip100_2p", "logistic1023_2p"):
        sp = WL.SPECS[name]
        n, d, ld = sp.n, sp.d, _ld(sp.d)
        X = torch.empty((n, ld), dtype=torch.float32, device="cuda")
        WL.device_normal((n, ld), sp.seed, out=X)
        ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:]
        res = torch.zeros(5, dtype=torch.float64, device="cuda")
        e = {"workload": name, "n": n, "d": d, "algorithmic_bytes": 4.0 * n * d}
        for key, call in (("consensus_error", lambda: P.consensus_error(X, n, d, res, workspace=ws, ld=ld)),
                          ("consensus_error_noalloc", lambda: P.consensus_error_noalloc(X, n, d, res, ld=ld))):
            for _ in range(warmup):
                call()
            with Timer(torch) as tm:
                for _ in range(steps):
                    call()
            ms = tm.event_ms / steps
            e[key] = {"ms_per_call": ms, "GBs": 4.0 * n * d / (ms * 1e-3) / 1e9, "frac": 4.0 * n * d / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        flat = X.reshape(-1)
        ms, gbs = probe(torch, P, (flat, None, None, flat, None), n * ld, 1, 0)
        e["read_only_probe_GBs"] = gbs
        if 4.0 * n * d < 64e6:
            e["bound"] = "launch latency (two launches, 17 MB): microseconds, not a bandwidth fraction"
        out.append(e)
        del X, ws
        torch.cuda.empty_cache()
    return out


def paper_lsq_runs(torch, P, Bn, name, runs=5):
    """The paper's least-squares experiment (Sec. 5) as the paper reports it: mean over `runs` independent
    runs (data, x(0) and gradient noise redrawn) of the final distance of the averaged model to x* and of
    the consensus error, after the workload's 200 iterations (windows of 20 at one step size through
    dsgd_ceca_run).  Not timed."""
    sp0 = WL.SPECS[name]
    n, d, N = sp0.n, sp0.d, sp0.N
    ld = _ld(d)
    tau = _tau(n)
    dist, cons, start = [], [], []
    for run in range(runs):
        sp = WL.for_run(sp0, run)
        Ah, bh, xs = WL.lsq_data(n, N, d, sp.seed, obs_noise=sp.obs_noise)
        A, t = torch.from_numpy(Ah).cuda(), torch.from_numpy(bh).cuda()
        K = sp.lr_decay_every
        idx = torch.from_numpy(WL.full_batch_indices(n, N)).cuda()[:1].repeat(K, 1, 1).contiguous()
        S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
        x0 = torch.from_numpy(WL.initial_state(n, d, sp.seed)).cuda()
        S[:n, :d] = x0
        S[n:, :d] = x0
        loss = lambda k: Bn.make_minibatch_loss(Bn.LOSS_LSQ, A, t, N, sp.B, grad_scale=sp.grad_scale,
                                                noise_std=sp.noise_std, seed=sp.seed, k=k)
        ws = torch.empty(P.dsgd_ceca_run_workspace_bytes(n, d, loss(0)) + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:]
        xs_d = torch.from_numpy(xs).cuda().double()
        start.append(float((S[:n, :d].double().mean(0) - xs_d).norm()))
        for w in range(sp.iters // K):
            P.dsgd_ceca_run(S, S, n, d, loss(w * K), idx, WL.step_size(sp, w * K), (w * K) % tau, K, sp.port,
                            workspace=ws, ld=ld)
        rep = consensus_report(torch, P, S[:n], n, d, ld)
        dist.append(float((S[:n, :d].double().mean(0) - xs_d).norm()))
        cons.append(rep["mean_distance_to_average"])
    return {"runs": runs, "iterations": sp0.iters, "mean_initial_distance_of_average_to_x_star": sum(start) / runs,
            "mean_final_distance_of_average_to_x_star": sum(dist) / runs,
            "mean_final_distance_to_average": sum(cons) / runs}


def run_mix(torch, P, Bn, n, d, steps, warmup):
    """Comparison-topology gossip (ring, static / one-peer exponential) at the sizes of the paper's consensus
    comparison: tau rounds fused into one ceca_mix_rounds call; 8 algorithmic bytes per agent-parameter
    for the whole call (x read once, written once)."""
    tau = _tau(n)
    ld = _ld(d)
    X = torch.empty((n, ld), dtype=torch.float32, device="cuda")
    WL.device_normal((n, ld), n, out=X)
    Y = torch.empty_like(X)
    kinds = {"ring": [P.ceca_topology_round(Bn.TOPO_RING, n)],
             "static_exp": [P.ceca_topology_round(Bn.TOPO_STATIC_EXP, n)],
             "one_peer_exp": [P.ceca_topology_round(Bn.TOPO_ONE_PEER_EXP, n, k) for k in range(tau)]}
    out = {"workload": f"mix{n}", "n": n, "d": d, "rounds_fused": tau, "algorithmic_bytes_per_agent_param": 8}
    # the consensus comparison itself (Sec. 5): residue max_i ||x_i - xbar|| / ||xbar|| after tau rounds, mean over
    # three independent draws of X(0) as in the paper; only CECA reaches the exact mean (not timed)
    resid = {k: 0.0 for k in list(kinds) + ["ceca_2p"]}
    for run in range(3):
        WL.device_normal((n, ld), n + 7919 * run, out=X)
        for kind, specs in kinds.items():
            P.ceca_mix_rounds(X, Y, n, d, specs, tau, ld=ld)
            resid[kind] += consensus_report(torch, P, Y, n, d, ld)["max_dev_over_mean_norm"] / 3
        P.ceca_average(X, Y, n, d, 2, ld=ld)
        resid["ceca_2p"] += consensus_report(torch, P, Y, n, d, ld)["max_dev_over_mean_norm"] / 3
    out["residue_after_tau_rounds_mean_of_3_runs"] = resid
    WL.device_normal((n, ld), n, out=X)
    for kind, specs in kinds.items():
        for _ in range(warmup):
            P.ceca_mix_rounds(X, Y, n, d, specs, tau, ld=ld)
        tm = Timer(torch)
        with tm:
            for _ in range(steps):
                P.ceca_mix_rounds(X, Y, n, d, specs, tau, ld=ld)
        ms = tm.event_ms / steps
        out[kind] = {"ms_per_call": ms, "GBs": 8.0 * n * d / (ms * 1e-3) / 1e9,
                     "agent_param_rounds_per_s": tau * n * d / (ms * 1e-3)}
    # graphs that are not shift-invariant go through neighbour tables (ceca_graph_rounds): a 2-D torus of
    # the same n with Metropolis weights, and the ring again as a table (same bits as the circulant kernel)
    rows = {130: 10, 1026: 27}.get(n, 1)
    for kind, edges in (("torus_graph", WL.edges_of("torus", n, rows)), ("ring_graph", WL.edges_of("ring", n))):
        tn, tw, ts = (torch.from_numpy(a[None]).cuda().contiguous() for a in WL.graph_table(n, edges))
        for _ in range(warmup):
            P.ceca_graph_rounds(X, Y, n, d, tn, tw, ts, tau, ld=ld)
        tm = Timer(torch)
        with tm:
            for _ in range(steps):
                P.ceca_graph_rounds(X, Y, n, d, tn, tw, ts, tau, ld=ld)
        ms = tm.event_ms / steps
        out[kind] = {"ms_per_call": ms, "GBs": 8.0 * n * d / (ms * 1e-3) / 1e9,
                     "agent_param_rounds_per_s": tau * n * d / (ms * 1e-3)}
    # CECA beside them: the same tau rounds on the same x reach the exact mean (ceca_average keeps the
    # auxiliary y in registers, so it also moves 8 bytes per agent-parameter)
    for port in (2, 1) if n % 2 == 0 else (2,):
        for _ in range(warmup):
            P.ceca_average(X, Y, n, d, port, ld=ld)
        tm = Timer(torch)
        with tm:
            for _ in range(steps):
                P.ceca_average(X, Y, n, d, port, ld=ld)
        ms = tm.event_ms / steps
        out[f"ceca_{port}p"] = {"ms_per_call": ms, "GBs": 8.0 * n * d / (ms * 1e-3) / 1e9,
                                "agent_param_rounds_per_s": tau * n * d / (ms * 1e-3)}
    # the simplest kernel with the same traffic (one streaming read, one streaming write per element)
    ms11, gb11 = probe(torch, P, (X.reshape(-1), None, None, Y.reshape(-1), None), n * ld, 1, 1)
    out["stream_probe_1r1w"] = {"ms_per_call": ms11, "GBs": gb11}
    return out


def measure(torch, P, Bn, name, steps, warmup):
    sp = WL.SPECS[name]
    fn = {"quad_center": run_quad, "none": run_gossip}.get(sp.loss, run_minibatch)
    tm, launches, (b_alg, b_model) = fn(torch, P, Bn, sp, steps, warmup)
    torch.cuda.empty_cache()
    ms = tm.wall_ms / steps
    ev_ms = tm.event_ms / steps
    units = sp.n * sp.d
    extra = {"graph_replay_ms_per_step": tm.graph_ms_per_step} if hasattr(tm, "graph_ms_per_step") else {}
    if hasattr(tm, "run_ms_per_step"):
        extra.update({"run_call_ms_per_step": tm.run_ms_per_step, "run_iterations_per_call": tm.run_iterations_per_call})
    extra.update(getattr(tm, "fused", {}))
    extra.update(getattr(tm, "probe", {}))
    if hasattr(tm, "final"):
        extra["consensus_after_timed_steps"] = tm.final
    if hasattr(tm, "frac"):
        extra["frac_per_step"] = tm.frac
    return {
        **extra,
        "workload": name, "n": sp.n, "d": sp.d, "port": sp.port, "loss": sp.loss, "steps": steps,
        "ms_per_step": ms, "event_ms_per_step": ev_ms, "kernels_per_step": launches,
        "agent_param_updates_per_s": units / (ms * 1e-3),
        "bytes_per_agent_param": b_alg, "bytes_per_agent_param_gather_model": b_model,
        "achieved_GBs": units * b_alg / (ev_ms * 1e-3) / 1e9,
        "gather_model_GBs": units * b_model / (ev_ms * 1e-3) / 1e9,
    }


def _shape_key(sh):
    return ",".join(str(sh[k]) for k in ("rows", "band", "wg_per_cu", "stretch"))


def measured_traffic(P, name, steps, warmup):
    """(mean HBM bytes per launch, note) from the committed rocprofv3 counter summary of this workload.
    The summary records the launch shape it was measured with (`shape_round0`, `shape_round`: rows in flight,
    band, workgroups per CU, stretch); a file without them, or with a shape other than the one the library
    now picks, is refused: its bytes may no longer describe the kernels timed here."""
    path = os.path.join(ROOT, "profiles", f"{name}_traffic.txt")
    if not os.path.exists(path):
        return None, "no counter summary committed for this workload"
    kv = {}
    with open(path) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split()
                kv[k] = v
    sp = WL.SPECS[name]
    tau = _tau(sp.n)
    ld = _ld(sp.d)
    kind = 1 if sp.loss == "quad_center" else (0 if sp.loss == "none" else 2)
    in_place = sp.port == 1
    now0 = _shape_key(P.ceca_describe_step_launch(sp.n, sp.d, ld, 0, sp.port, kind, in_place))
    now1 = _shape_key(P.ceca_describe_step_launch(sp.n, sp.d, ld, 1 % tau, sp.port, kind, in_place))
    if kv.get("shape_round0") != now0 or kv.get("shape_round") != now1:
        return None, (f"stale: the summary was measured with launch shapes {kv.get('shape_round0')} / {kv.get('shape_round')}, "
                      f"the library now picks {now0} / {now1}")
    fs, wsc = float(kv["fetch_scale"]), float(kv["write_scale"])
    if "step_fetch_kib" in kv:
        # minibatch workloads: the counters summed over the launches of one step, reported per launch
        return (1024.0 * (float(kv["step_fetch_kib"]) * fs + float(kv["step_write_kib"]) * wsc) / float(kv["launches_per_step"]),
                "FETCH_SIZE / WRITE_SIZE summary, same launch shapes")
    r0 = float(kv["round0_fetch_kib"]) * fs + float(kv["round0_write_kib"]) * wsc
    rr = float(kv["round_fetch_kib"]) * fs + float(kv["round_write_kib"]) * wsc
    rounds = [k % tau for k in range(warmup, warmup + steps)]
    return 1024.0 * sum(r0 if r == 0 else rr for r in rounds) / len(rounds), "FETCH_SIZE / WRITE_SIZE summary, same launch shapes"


# ---------------------------------------------------------------------------------------------
# CPU baseline: the fp64 numpy oracle as it stands, on a bounded sample of the workload, on one thread and on
# all host cores.  Runs before this process touches the GPU; the workers are fresh interpreters (spawn).
# ---------------------------------------------------------------------------------------------
def _cpu_sample(name, block, target_s, barrier=None):
    """One worker's share: the oracle on block number `block` of the sample, for about target_s seconds.
    Returns (agent-parameter updates done, seconds, iterations, description of the block)."""
    from oracle import ceca as OC
    from oracle import losses as OL

    sp = WL.SPECS[name]
    n, port = sp.n, sp.port
    if sp.loss in ("quad_center", "none"):
        # columns are independent instances of the recursion: a block is 2^18 of them, all agents
        width = min(sp.d, 1 << 18)
        c0 = (block * width) % max(sp.d - width + 1, 1)
        cols = np.arange(c0, c0 + width, dtype=np.int64)
        if sp.loss == "quad_center":
            grad = OL.make_quad_center_grad(WL.quad_centers(n, width, sp.seed + 1000 * block), sp.noise_std, sp.seed, columns=cols)
            x = y = np.zeros((n, width))
        else:
            grad = None
            x = y = WL.initial_state(n, width, sp.seed + 1000 * block).astype(np.float64)
        what = f"{width} of {sp.d} columns, all {n} agents"
    else:
        # minibatch losses couple the columns: keep d and B, cut the agent count and the sample pool; a block
        # is an independent replica drawn with its own seed
        n = min(n, 127)
        N = min(sp.N, 64)
        seed = sp.seed + 1000 * block
        if name.startswith("logistic1023"):
            A, t, _ = WL.logistic_data_sparse(n, N, sp.d, seed)
        elif sp.loss == "lsq":
            A, t, _ = WL.lsq_data(n, N, sp.d, seed)
        else:
            A, t, _ = WL.logistic_data_hetero(n, N, sp.d, seed)
        B = min(sp.B, N)
        idx = WL.full_batch_indices(n, N) if sp.B == sp.N else WL.batch_indices(n, N, B, 256, seed)
        grad = OL.make_minibatch_grad(sp.loss, A, t, idx, grad_scale=sp.grad_scale, noise_std=sp.noise_std,
                                      seed=sp.seed)
        x = y = np.zeros((n, sp.d))
        width = sp.d
        what = f"{n} of {sp.n} agents, {N} of {sp.N} samples each, all {sp.d} columns"
    tau = _tau(n)
    if barrier is not None:
        try:
            barrier.wait(timeout=60.0)      # all workers start their timed loops together
        except Exception:
            pass                            # a worker that never arrived must not stop the others
    t0 = time.perf_counter()
    iters = 0
    while True:
        if grad is None:
            x, y = OC.gossip_round(x, y, iters % tau, port, store32=True)
        else:
            x, y = OC.dsgd_ceca_step(x, y, iters, port, WL.step_size(sp, iters), grad, store32=True)
        iters += 1
        el = time.perf_counter() - t0
        if el > target_s:
            break
    return float(n) * width * iters, el, iters, what


def _cpu_worker(name, block, target_s, barrier, queue):
    try:                                    # one thread per worker, also inside the BLAS library
        import threadpoolctl
        threadpoolctl.threadpool_limits(1)
    except Exception:
        pass
    try:
        queue.put((block,) + _cpu_sample(name, block, target_s, barrier))
    except Exception as e:                  # the parent counts the workers that report
        queue.put((block, None, repr(e)))


def cpu_baseline(sp, target_s=10.0):
    """The oracle timed twice on bounded samples of the workload: one thread (the oracle is plain numpy: its
    elementwise code and its small per-agent matrix products run on one thread), then one worker process
    per host core available to this run, each on its own block of the sample, started together.  The
    workers are fresh interpreters (spawn) started before this process touches the GPU; every wait on them
    has a deadline, and a worker that fails only lowers the count of cores reported."""
    import multiprocessing as mp
    import queue as queue_mod

    units1, el1, it1, what = _cpu_sample(sp.name, 0, target_s)
    single = {"value": units1 / el1, "cores": 1, "sample": f"{it1} iterations of {sp.name} on {what}; {el1:.1f} s"}
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    # a one-GPU machine gives a run 16 cores' worth whatever the machine has
    workers = max(1, min(avail, 16))
    ctx = mp.get_context("spawn")
    barrier = ctx.Barrier(workers)
    q = ctx.Queue()
    procs = [ctx.Process(target=_cpu_worker, args=(sp.name, j, target_s, barrier, q), daemon=True) for j in range(workers)]
    for pr in procs:
        pr.start()
    res = []
    deadline = time.perf_counter() + target_s + 120.0
    while len(res) < workers and time.perf_counter() < deadline:
        try:
            r = q.get(timeout=1.0)
        except queue_mod.Empty:
            if not any(pr.is_alive() for pr in procs):
                break
            continue
        res.append(r)
    for pr in procs:
        pr.join(timeout=5.0)
        if pr.is_alive():
            pr.terminate()
    good = [r for r in res if r[1] is not None]
    base = {"unit": "agent-param updates/s", "kind": "oracle", "single_thread": single,
            "host_cpu_count": os.cpu_count(), "host_cpus_available": avail}
    if not good:
        return {**base, "value": single["value"], "cores": 1,
                "sample": single["sample"] + "; the all-core leg did not finish: " + "; ".join(str(r[2]) for r in res if r[1] is None)}
    units = sum(r[1] for r in good)
    el = max(r[2] for r in good)
    its = [r[3] for r in good]
    return {**base, "value": units / el, "cores": len(good),
            "sample": f"{len(good)} worker processes, each {min(its)}-{max(its)} iterations of {sp.name} on its own block of "
                      f"{good[0][4]}; fp64 numpy oracle, {el:.1f} s; in all {units / (sp.n * sp.d):.2f} full-width iterations' worth"}


def config_entry(res, sp):
    """One compact line of the `configs` block from a measure() result."""
    hbm = sp.loss in ("quad_center", "none") or sp.name.startswith("logistic1023")
    e = {"workload": sp.name, "n": sp.n, "d": sp.d, "port": sp.port, "loss": sp.loss, "steps": res["steps"],
         "ms_per_step": res["ms_per_step"], "us_per_iteration": res["ms_per_step"] * 1e3,
         "kernels_per_step": res["kernels_per_step"], "agent_param_updates_per_s": res["agent_param_updates_per_s"]}
    if hbm:
        e.update({"bound": "hbm", "bytes_per_agent_param": res["bytes_per_agent_param"],
                  "algorithmic_bytes_per_step": res["bytes_per_agent_param"] * sp.n * sp.d,
                  "achieved_GBs": res["achieved_GBs"], "frac": res["achieved_GBs"] / HBM_PEAK_GBS})
    else:
        e["bound"] = "launch latency (no bandwidth fraction is claimed)"
    for k in ("graph_replay_ms_per_step", "run_call_ms_per_step", "run_iterations_per_call", "fused_rounds", "fused_ms",
              "fused_GBs_on_12B", "fused_probe_1r2w_ms", "average_ms", "average_GBs_on_8B", "average_probe_1r1w_ms",
              "frac_per_step", "consensus_after_timed_steps"):
        if k in res:
            e[k] = res[k]
    if "run_call_ms_per_step" in res:
        # the same iterations through dsgd_ceca_run (one call per window): the fastest way this library runs them
        e["run_call_agent_param_updates_per_s"] = sp.n * sp.d / (res["run_call_ms_per_step"] * 1e-3)
        if hbm:
            e["run_call_frac"] = res["bytes_per_agent_param"] * sp.n * sp.d / (res["run_call_ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="quad31_2p", choices=sorted(WL.SPECS))
    ap.add_argument("--others", action="store_true", help="also time the remaining workloads in full (reported under 'others')")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the short timings of the other configurations (the `configs` block of the default run)")
    ap.add_argument("--consensus-only", action="store_true",
                    help="time only consensus_error at the configuration sizes and exit")
    ap.add_argument("--mix-only", action="store_true",
                    help="time only the comparison-topology gossip rounds (n = 130 and n = 1026) and exit")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--eager-only", action="store_true",
                    help="minibatch workloads: time the eager steps only (no HIP-graph replay, no multi-iteration calls); "
                         "for hardware-counter passes")
    ap.add_argument("--no-graph", action="store_true", help="minibatch workloads: skip only the HIP-graph replay leg")
    ap.add_argument("--copy-probe", action="store_true",
                    help="first run one plain 1 GiB device copy (calibrates rocprofv3 byte counters)")
    ap.add_argument("--write-data", metavar="FILE", help="minibatch workloads: draw the inputs, save them as FILE.A.npy / FILE.t.npy and exit")
    ap.add_argument("--data-file", metavar="FILE", help="minibatch workloads: load the inputs an earlier --write-data run saved")
    args = ap.parse_args()
    global EAGER_ONLY, NO_GRAPH, DATA_FILE, WRITE_DATA
    EAGER_ONLY = args.eager_only
    NO_GRAPH = args.no_graph
    DATA_FILE = args.write_data or args.data_file
    WRITE_DATA = bool(args.write_data)
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (all agents are simulated on one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    sp = WL.SPECS[args.workload]
    profiling = args.eager_only or args.no_graph or args.copy_probe or WRITE_DATA or bool(args.data_file)

    # the CPU leg comes first: its worker processes are started from a process that holds no GPU state
    cpu = None
    if not (args.no_cpu or args.mix_only or args.consensus_only or profiling):
        cpu = cpu_baseline(sp)

    import torch

    import paper_2306_00256_amd as P
    from paper_2306_00256_amd import binding as Bn

    P.lib()     # raises if the HIP library is missing: there is no fallback path
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    def copy_probe():
        # a plain copy of known size (1 GiB read, 1 GiB written): calibrates the byte counters of a --pmc run
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.mix_only:
        if args.copy_probe:
            copy_probe()
        print(json.dumps({"mix": [run_mix(torch, P, Bn, 130, 1 << 20, args.steps, args.warmup),
                                  run_mix(torch, P, Bn, 1026, 1 << 17, args.steps, args.warmup)]}), flush=True)
        return

    if args.consensus_only:
        if args.copy_probe:
            copy_probe()
        print(json.dumps({"consensus": run_consensus(torch, P, Bn, args.steps, args.warmup)}), flush=True)
        return

    if args.copy_probe:
        copy_probe()

    main_res = measure(torch, P, Bn, args.workload, args.steps, args.warmup)
    traffic, traffic_note = measured_traffic(P, args.workload, args.steps, args.warmup)
    out = {
        "metric": "agent-param updates/s per DSGD-CECA round",
        "value": main_res["agent_param_updates_per_s"],
        "unit": "agent-param updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_agents": sp.n, "d": sp.d, "port": sp.port, "loss": sp.loss,
                   "lr": sp.lr, "ld": _ld(sp.d), "state_bytes": 2 * sp.n * _ld(sp.d) * 4},
        "roofline": {
            "bound": "hbm",
            "achieved": main_res["achieved_GBs"],
            "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": main_res["achieved_GBs"] / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": traffic_note,
            "algorithmic_bytes_per_launch": main_res["bytes_per_agent_param"] * sp.n * sp.d
            / main_res["kernels_per_step"],
            "bytes_per_agent_param": main_res["bytes_per_agent_param"],
            "kernel_ms": main_res["event_ms_per_step"] / main_res["kernels_per_step"],
            "gather_model_GBs": main_res["gather_model_GBs"],
            # spread of the per-step fraction of peak (each step against its own round's bytes), from a second
            # pass over the same steps with an event after every launch
            "frac_per_step": main_res.get("frac_per_step"),
            # the simplest elementwise kernel with the same reads and writes per element, timed in this run:
            # a full round's mix, round 0's mix, and the full round's mix in place
            "stream_probe_GBs": main_res.get("stream_probe_GBs"),
            "stream_probe_ms": main_res.get("stream_probe_ms"),
            "stream_probe_round0_GBs": main_res.get("stream_probe_round0_GBs"),
            "stream_probe_round0_ms": main_res.get("stream_probe_round0_ms"),
            "stream_probe_in_place_GBs": main_res.get("stream_probe_in_place_GBs"),
        },
    }
    details = {k: main_res[k] for k in ("graph_replay_ms_per_step", "run_call_ms_per_step", "run_iterations_per_call",
                                        "fused_rounds", "fused_ms", "fused_GBs_on_12B", "fused_probe_1r2w_ms", "average_ms",
                                        "average_GBs_on_8B", "average_probe_1r1w_ms", "caller_gradient_step_ms",
                                        "max_dev_over_mean_norm_after_round", "consensus_after_timed_steps")
               if k in main_res}
    if details:
        out["details"] = details
    if "fused_iterations_per_call" in main_res:
        # not the headline: `value` is the one-launch-per-iteration path that the metric names
        out["fused_iterations"] = {k: main_res[k] for k in ("fused_iterations_per_call", "fused_ms_per_iteration",
                                                             "fused_agent_param_updates_per_s")}
        out["fused_iterations"]["speedup_over_value"] = main_res["fused_agent_param_updates_per_s"] / out["value"]
    comp = None
    if args.workload == "quad31_2p" and not args.others and not profiling:
        # the configuration names one-port CECA, which needs an even number of agents: the same workload at
        # n = 30 with one port (in place, closed pairs) beside the two-port run at the stated n = 31
        comp = measure(torch, P, Bn, "quad30_1p", args.steps, args.warmup)
        out["companion_1p"] = {"workload": "quad30_1p", "n_agents": 30, "port": 1, "ms_per_step": comp["ms_per_step"],
                               "value": comp["agent_param_updates_per_s"], "achieved_GBs": comp["achieved_GBs"],
                               "frac": comp["achieved_GBs"] / HBM_PEAK_GBS, "frac_per_step": comp.get("frac_per_step")}
    if args.workload == "quad31_2p" and not (args.others or args.no_configs or profiling):
        # every configuration in the one line the default run prints: the five stated ones (the two that ask
        # for one port at an odd n appear at both readings) and the paper's own least-squares experiment
        cfgs = [config_entry(main_res, sp)]
        if comp is not None:
            cfgs.append(config_entry(comp, WL.SPECS["quad30_1p"]))
        for name in ("gossip100_1p", "gossip100_2p", "logistic1023_2p", "logistic6_2p", "lsq5_2p", "lsq6_1p",
                     "paperlsq258_1p", "paperlsq258_2p"):
            sp_o = WL.SPECS[name]
            k = 70 if sp_o.loss == "none" else 200
            cfgs.append(config_entry(measure(torch, P, Bn, name, k, 5), sp_o))
            if name.startswith("paperlsq258"):
                cfgs[-1]["mean_over_5_runs"] = paper_lsq_runs(torch, P, Bn, name)
        out["configs"] = cfgs
        out["consensus"] = run_consensus(torch, P, Bn)
        # the consensus comparison at the paper's sizes (Sec. 5): ring, static and one-peer exponential gossip,
        # gossip over a torus, CECA's exact averaging and the streaming probe with their traffic, tau rounds per call
        torch.cuda.empty_cache()
        out["mix"] = [run_mix(torch, P, Bn, 130, 1 << 20, 10, 2), run_mix(torch, P, Bn, 1026, 1 << 17, 10, 2)]
    if args.others:
        out["others"] = []
        for name in sorted(WL.SPECS):
            if name == args.workload:
                continue
            sp_o = WL.SPECS[name]
            k = 50 if sp_o.loss in ("quad_center",) else (70 if sp_o.loss == "none" else 200)
            out["others"].append(measure(torch, P, Bn, name, k, 5))
        out["others"].append(run_mix(torch, P, Bn, 130, 1 << 20, 20, 3))
        out["others"].append(run_mix(torch, P, Bn, 1026, 1 << 17, 20, 3))
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
