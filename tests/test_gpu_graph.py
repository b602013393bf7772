"""HIP-graph capture of the launch-bound training loop: every replay must equal the eager result.

The library only launches kernels on the caller's stream (no allocation, no memset, no synchronization),
so a caller may capture a window of iterations and replay it."""
import numpy as np
import pytest

import workloads as WL
from oracle import schedule as OS
from gpu_util import make_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


@pytest.mark.parametrize("name", ["lsq6_1p", "lsq5_2p"])
def test_graph_replays_equal_eager(env, name):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    sp = WL.SPECS[name]
    n, d, N, B, port = sp.n, sp.d, sp.N, sp.B, sp.port
    tau = OS.num_rounds(n)
    window = 2 * tau                                   # even, so two-port ping-pong buffers end where they began
    A, b, _ = WL.lsq_data(n, N, d, sp.seed)
    idx = torch.from_numpy(WL.batch_indices(n, N, B, window, sp.seed)).cuda()
    Ad, bd = torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda()
    loss = Bn.make_minibatch_loss(Bn.LOSS_LSQ, Ad, bd, N, B)
    ws = torch.empty(P.dsgd_ceca_workspace_bytes(n, d, loss), dtype=torch.uint8, device="cuda")
    x0 = 0.1 * WL.initial_state(n, d, sp.seed)

    def run_window(S, T):
        for k in range(window):
            P.dsgd_ceca_step(S, T, n, d, loss, idx[k], sp.lr, k % tau, port, workspace=ws)
            if port == 2:
                S, T = T, S

    replays = 4
    # eager reference: the same window `replays` times
    S = make_state(torch, x0)
    T = S if port == 1 else make_state(torch, np.zeros_like(x0))
    eager = []
    for _ in range(replays):
        run_window(S, T)
        torch.cuda.synchronize()
        eager.append(S.cpu().numpy().copy())

    S2 = make_state(torch, x0)
    T2 = S2 if port == 1 else make_state(torch, np.zeros_like(x0))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_window(S2, T2)                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    S2.copy_(make_state(torch, x0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_window(S2, T2)
    S2.copy_(make_state(torch, x0))                     # capture does not execute: restore the start state
    for rep in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        scratch = torch.randn(1024, device="cuda").sum().item()      # unrelated eager work between replays
        assert np.isfinite(scratch)
        assert np.array_equal(S2.cpu().numpy(), eager[rep]), rep


def test_graph_of_the_multi_iteration_calls(env):
    """dsgd_ceca_run (fused gradient + combine kernels), dsgd_ceca_steps, ceca_gossip_rounds,
    ceca_mix_rounds and ceca_state_consensus captured in one graph: every replay equals the eager run."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, N, B, iters, port = 130, 2048, 8, 6, 5, 2
    A, t, _ = WL.logistic_data_sparse(n, N, d, seed=2, density=0.5)
    idx = torch.from_numpy(WL.batch_indices(n, N, B, iters, seed=2)).cuda()
    Ad, td = torch.from_numpy(A).cuda(), torch.from_numpy(t).cuda()
    loss = Bn.make_minibatch_loss(Bn.LOSS_LOGISTIC, Ad, td, N, B, noise_std=0.01, seed=3)
    wsr = torch.empty(P.dsgd_ceca_run_workspace_bytes(n, d, loss) + 256, dtype=torch.uint8, device="cuda")
    wsr = wsr[(-wsr.data_ptr()) % 256:]
    wsc = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
    wsc = wsc[(-wsc.data_ptr()) % 256:]
    c = torch.from_numpy(WL.quad_centers(n, d, 4)).cuda()
    qloss = Bn.make_quad_center_loss(c, 0.01, 5, 0)
    ring = [P.ceca_topology_round(Bn.TOPO_RING, n)]
    x0 = 0.1 * WL.initial_state(n, d, 6)
    tau = OS.num_rounds(n)

    def window(S, out):
        P.dsgd_ceca_run(S, S, n, d, loss, idx, 0.01, 0, iters, port, workspace=wsr)
        P.dsgd_ceca_steps(S, S, n, d, qloss, 0.05, iters % tau, 3, port)
        P.ceca_mix_rounds(S[:n], S[:n], n, d, ring, 2)
        P.ceca_gossip_rounds(S, S, n, d, 2, port)
        P.ceca_state_consensus(S, n, d, out, workspace=wsc)

    replays = 3
    S = make_state(torch, x0)
    out = torch.zeros(11, dtype=torch.float64, device="cuda")
    eager = []
    for _ in range(replays):
        window(S, out)
        torch.cuda.synchronize()
        eager.append((S.cpu().numpy().copy(), out.cpu().numpy().copy()))

    S2 = make_state(torch, x0)
    out2 = torch.zeros(11, dtype=torch.float64, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        window(S2, out2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    S2.copy_(make_state(torch, x0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        window(S2, out2)
    S2.copy_(make_state(torch, x0))
    for rep in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(torch.randn(1024, device="cuda").sum().item())      # unrelated eager work in between
        assert np.array_equal(S2.cpu().numpy(), eager[rep][0]), rep
        assert np.array_equal(out2.cpu().numpy(), eager[rep][1]), rep


def test_graph_of_the_wide_workgroup_kernels(env):
    """More than 1000 agents: the fused rounds, fused iterations and mixing kernels run 512- and 1024-thread
    workgroups with more than 64 KB of LDS each (asked for per launch); captured in a graph, every replay
    equals the eager run."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, port = 1026, 132, 2
    tau = OS.num_rounds(n)
    c = torch.from_numpy(WL.quad_centers(n, d, 4)).cuda()
    qloss = Bn.make_quad_center_loss(c, 0.01, 5, 0)
    one_peer = [P.ceca_topology_round(Bn.TOPO_ONE_PEER_EXP, n, k) for k in range(tau)]
    x0 = WL.initial_state(n, d, 8)

    def window(S):
        P.dsgd_ceca_steps(S, S, n, d, qloss, 0.05, 0, 4, port)
        P.ceca_mix_rounds(S[:n], S[:n], n, d, one_peer, 3)
        P.ceca_gossip_rounds(S, S, n, d, tau - 1, port)
        P.ceca_average(S[n:], S[n:], n, d, port)

    replays = 3
    S = make_state(torch, x0)
    eager = []
    for _ in range(replays):
        window(S)
        torch.cuda.synchronize()
        eager.append(S.cpu().numpy().copy())
    S2 = make_state(torch, x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        window(S2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    S2.copy_(make_state(torch, x0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        window(S2)
    S2.copy_(make_state(torch, x0))
    for rep in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(torch.randn(1024, device="cuda").sum().item())      # unrelated eager work in between
        assert np.array_equal(S2.cpu().numpy(), eager[rep]), rep


def test_concurrent_calls_on_two_streams_from_two_threads(env):
    """The library keeps no per-call state (no global scratch): two host threads driving different problems
    on their own streams at the same time get the results of running them one after the other."""
    import threading
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    jobs = []
    for n, d, port, seed in [(100, 4096 + 4, 2, 1), (30, 8192, 1, 2)]:
        x0 = WL.initial_state(n, d, seed)
        c = torch.from_numpy(WL.quad_centers(n, d, seed)).cuda()
        jobs.append((n, d, port, x0, c))

    def work(job, stream, out):
        n, d, port, x0, c = job
        tau = OS.num_rounds(n)
        with torch.cuda.stream(stream):
            S = make_state(torch, x0)
            T = S if port == 1 else torch.empty_like(S)
            for k in range(3 * tau):
                P.dsgd_ceca_step(S, T, n, d, Bn.make_quad_center_loss(c, 0.01, 7, k), None, 0.1, k % tau, port, stream=stream)
                S, T = T, S
            P.ceca_gossip_rounds(S, S, n, d, tau + 1, port, stream=stream)
            stream.synchronize()
            out.append(S.cpu().numpy().copy())

    serial = []
    for job in jobs:
        out = []
        work(job, torch.cuda.current_stream(), out)
        serial.append(out[0])
    torch.cuda.synchronize()
    for _ in range(3):
        outs = [[], []]
        threads = [threading.Thread(target=work, args=(jobs[i], torch.cuda.Stream(), outs[i])) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        for i in range(2):
            assert np.array_equal(outs[i][0], serial[i]), i


def test_graph_of_a_run_on_the_two_pass_gradient(env):
    """dsgd_ceca_run on a shape whose gradient takes two passes (the state alternates between S_out and a copy
    in the workspace): captured once, every replay continues the eager trajectory."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, N, B, iters, port = 6, 10000, 20, 32, 5, 2
    A, t, _ = WL.logistic_data_sparse(n, N, d, seed=5, density=0.5)
    idx = torch.from_numpy(WL.batch_indices(n, N, B, iters, seed=5)).cuda()
    Ad, td = torch.from_numpy(A).cuda(), torch.from_numpy(t).cuda()
    loss = Bn.make_minibatch_loss(Bn.LOSS_LOGISTIC, Ad, td, N, B)
    ws = torch.empty(P.dsgd_ceca_run_workspace_bytes(n, d, loss) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    x0 = 0.1 * WL.initial_state(n, d, 6)
    replays = 3
    S = make_state(torch, x0)
    eager = []
    for _ in range(replays):
        P.dsgd_ceca_run(S, S, n, d, loss, idx, 0.01, 0, iters, port, workspace=ws)
        torch.cuda.synchronize()
        eager.append(S.cpu().numpy().copy())
    S2 = make_state(torch, x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        P.dsgd_ceca_run(S2, S2, n, d, loss, idx, 0.01, 0, iters, port, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    S2.copy_(make_state(torch, x0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        P.dsgd_ceca_run(S2, S2, n, d, loss, idx, 0.01, 0, iters, port, workspace=ws)
    S2.copy_(make_state(torch, x0))
    for rep in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(torch.randn(1024, device="cuda").sum().item())      # unrelated eager work in between
        assert np.array_equal(S2.cpu().numpy(), eager[rep]), rep
