"""GPU parity at the size limits of the fused kernels: the largest agent counts one workgroup's
registers take (4096) and the first ones beyond, where the calls fall back to one launch per round."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as OC
from oracle import losses as OL
from oracle import schedule as OS
from oracle import topologies as OT
from gpu_util import make_state, rel_err, split_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


@pytest.mark.parametrize("n,port", [(4095, 2), (4096, 1), (4096, 2), (4097, 2), (4098, 1), (5000, 2)])
def test_fused_rounds_around_the_agent_limit(env, n, port):
    torch, P = env
    d = 37
    tau = OS.num_rounds(n)
    x0 = WL.initial_state(n, d, seed=n)
    S = make_state(torch, x0, y0=np.full_like(x0, np.nan))
    T = make_state(torch, np.zeros_like(x0))
    P.ceca_gossip_rounds(S, T, n, d, tau + 1, port)
    gx, gy = split_state(T, n, d)
    x, y = OC.run(x0, port, 0.0, None, tau + 1, store32=True)
    assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5
    mean = x0.astype(np.float64).mean(axis=0)
    assert np.abs(gx - mean).max() <= 1e-6 and np.abs(gy - mean).max() <= 1e-6     # Lemma 4.2: both at the mean
    # same bits as single rounds
    A = make_state(torch, x0)
    B = make_state(torch, np.zeros_like(x0))
    for r in range(tau + 1):
        P.ceca_gossip_round(A, B, n, d, r % tau, port)
        A, B = B, A
    ax, ay = split_state(A, n, d)
    assert np.array_equal(ax, gx) and np.array_equal(ay, gy)


@pytest.mark.parametrize("n,port", [(4096, 1), (4097, 2)])
def test_fused_iterations_around_the_agent_limit(env, n, port):
    """4096 agents still fit one workgroup's registers, 4097 do not.  With tile rows this narrow the library
    fuses only long runs (15 iterations here) and takes short ones (5) step by step; setting the rows
    option makes it fuse those too.  All give the same bits, and the oracle's values."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    d, seed, lr, std = 21, 9, 0.1, 0.01
    c = WL.quad_centers(n, d, seed)
    cdev = torch.from_numpy(c).cuda()
    x0 = WL.initial_state(n, d, seed)
    for steps in (5, 15):
        outs = []
        try:
            for rows in (0, 16):
                P.ceca_set_option(Bn.OPT_ROWS, rows)
                A = make_state(torch, x0)
                B = make_state(torch, np.zeros_like(x0))
                P.dsgd_ceca_steps(A, B, n, d, Bn.make_quad_center_loss(cdev, std, seed, 2), lr, 2, steps, port)
                outs.append(B)
        finally:
            P.ceca_set_option(Bn.OPT_ROWS, 0)
        assert torch.equal(outs[0], outs[1])
        gx, gy = split_state(outs[0], n, d)
        x, y = OC.run(x0, port, lr, OL.make_quad_center_grad(c, std, seed), steps, store32=True, k0=2)
        assert max(rel_err(gx, x)) <= 1e-4 and max(rel_err(gy, y)) <= 1e-4


def test_mixing_rounds_at_the_agent_limit(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d = 4096, 29
    x0 = WL.initial_state(n, d, seed=4)
    X = torch.from_numpy(x0).cuda()
    for kind, want in [(Bn.TOPO_STATIC_EXP, [OT.static_exponential(n)]), (Bn.TOPO_RING, [OT.ring(n)])]:
        Y = torch.empty_like(X)
        P.ceca_mix_rounds(X, Y, n, d, [P.ceca_topology_round(kind, n)], 3)
        assert max(rel_err(Y.cpu().numpy(), OT.run(x0, want, 3))) <= 1e-5
    with pytest.raises(P.CecaError) as e:
        P.ceca_mix_rounds(X, X, 4097, d, [P.ceca_topology_round(Bn.TOPO_RING, 4097)], 1)
    assert e.value.code == Bn.CECA_EINVAL


@pytest.mark.parametrize("n,port", [(70001, 2), (70000, 1), (131072, 2)])
def test_very_many_agents(env, n, port):
    """More agents than any grid dimension but the first can index (65535): gossip rounds, fused rounds
    (one launch per round at this size), the consensus observables and the state consensus call."""
    torch, P = env
    from oracle import consensus as OCONS
    d = 6
    tau = OS.num_rounds(n)
    x0 = WL.initial_state(n, d, seed=n % 1000)
    S = make_state(torch, x0)
    T = make_state(torch, np.zeros_like(x0))
    x = y = x0.astype(np.float64)
    for r in range(3):
        P.ceca_gossip_round(S, T, n, d, r, port)
        S, T = T, S
        x, y = OC.gossip_round(x, y, r, port, store32=True)
    gx, gy = split_state(S, n, d)
    assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5
    F = make_state(torch, x0)
    P.ceca_gossip_rounds(F, F, n, d, tau, port)
    fx, _ = split_state(F, n, d)
    mean = x0.astype(np.float64).mean(axis=0)
    assert np.abs(fx - mean).max() <= 5e-7          # inputs are N(0, 1): fp32 rounding of the early rounds
    ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    out = torch.zeros(11, dtype=torch.float64, device="cuda")
    P.ceca_state_consensus(S, n, d, out, workspace=ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = OCONS.state_consensus(gx, gy)
    assert abs(got[0] - want["x"]["frob2"]) <= 1e-10 * want["x"]["frob2"]
    assert abs(got[5] - want["y"]["frob2"]) <= 1e-10 * want["y"]["frob2"]
    assert abs(got[10] - want["phi2"]) <= 1e-10 * want["phi2"]


def test_minibatch_losses_refuse_more_than_65535_agents(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, N, B = 65536, 4, 2, 1
    A = torch.zeros((n, N, d), dtype=torch.float32, device="cuda")
    t = torch.zeros((n, N), dtype=torch.float32, device="cuda")
    idx = torch.zeros((n, B), dtype=torch.int32, device="cuda")
    S = torch.zeros((2 * n, d), dtype=torch.float32, device="cuda")
    loss = Bn.make_minibatch_loss(Bn.LOSS_LSQ, A, t, N, B)
    ws = torch.empty(max(P.dsgd_ceca_workspace_bytes(n, d, loss), 256), dtype=torch.uint8, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.dsgd_ceca_step(S, S, n, d, loss, idx, 0.1, 0, 2, workspace=ws)
    assert e.value.code == Bn.CECA_EINVAL


def test_xcd_tile_order_does_not_change_results(env):
    """Many narrow tiles (more than 1024 agents-wide tiles of 64-byte rows): the XCD-contiguous workgroup
    order and the plain order give the same bits in the fused rounds, fused iterations and mixing kernels."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, port = 1026, 16 * 1500 + 4, 1
    x0 = WL.initial_state(n, d, seed=3)
    c = torch.from_numpy(WL.quad_centers(n, d, 4)).cuda()
    ring = [P.ceca_topology_round(Bn.TOPO_RING, n)]
    outs = []
    try:
        for order in (1, 0):
            P.ceca_set_option(Bn.OPT_XCD_TILE_ORDER, order)
            S = make_state(torch, x0)
            P.ceca_gossip_rounds(S, S, n, d, 5, port)
            P.dsgd_ceca_steps(S, S, n, d, Bn.make_quad_center_loss(c, 0.01, 1, 0), 0.1, 5 % OS.num_rounds(n), 3, port)
            P.ceca_mix_rounds(S[:n], S[:n], n, d, ring, 2)
            outs.append(S.clone())
    finally:
        P.ceca_set_option(Bn.OPT_XCD_TILE_ORDER, 1)
    assert torch.equal(outs[0], outs[1])
    x, y = OC.run(x0, port, 0.0, None, 5, store32=True)
    ref = make_state(torch, x0)
    P.ceca_gossip_rounds(ref, ref, n, d, 5, port)
    gx, gy = split_state(ref, n, d)
    assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5


def test_more_rounds_than_one_kernel_takes(env):
    """ceca_gossip_rounds beyond 64 rounds (several kernels of whole cycles, in place after the first) and
    ceca_mix_rounds with hundreds of rounds in one kernel: same bits as the calls split into shorter runs,
    and the oracle's values."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    # tau = 5 does not divide 64 (pieces of 60 rounds), out of place, ragged columns, both ports
    for n2, port2 in [(20, 2), (18, 1)]:
        d2, rounds = 1027, 131
        tau2 = OS.num_rounds(n2)
        z0 = WL.initial_state(n2, d2, seed=9)
        src = make_state(torch, z0)
        keep = src.clone()
        dst = torch.full_like(src, float("nan"))
        P.ceca_gossip_rounds(src, dst, n2, d2, rounds, port2)
        assert torch.equal(src, keep)
        ref = make_state(torch, z0)
        for t in range(rounds):
            P.ceca_gossip_round(ref, ref, n2, d2, t % tau2, port2)
        assert torch.equal(dst, ref), (n2, port2)
        x, y = OC.run(z0, port2, 0.0, None, rounds, store32=True)
        gx, gy = split_state(dst, n2, d2)
        assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5
    n, d, port = 12, 300, 2
    tau = OS.num_rounds(n)
    x0 = WL.initial_state(n, d, seed=8)
    A = make_state(torch, x0)
    P.ceca_gossip_rounds(A, A, n, d, 70, port)
    B = make_state(torch, x0)
    P.ceca_gossip_rounds(B, B, n, d, 64, port)
    for t in range(64, 70):
        P.ceca_gossip_round(B, B, n, d, t % tau, port)
    assert torch.equal(A, B)
    x, y = OC.run(x0, port, 0.0, None, 70, store32=True)
    gx, gy = split_state(A, n, d)
    assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5
    ring = [P.ceca_topology_round(Bn.TOPO_RING, n)]
    X = torch.from_numpy(x0).cuda()
    Y = X.clone()
    P.ceca_mix_rounds(X, X, n, d, ring, 300)
    for _ in range(3):
        P.ceca_mix_rounds(Y, Y, n, d, ring, 100)
    assert torch.equal(X, Y)
    want = OT.run(x0, [OT.ring(n)], 300)
    assert max(rel_err(X.cpu().numpy(), want)) <= 1e-4


@pytest.mark.parametrize("n,port", [(2, 2), (6, 1), (9, 2), (31, 2), (100, 1), (145, 2), (1026, 1), (1153, 2), (2050, 1), (4096, 2)])
def test_workgroup_widths_of_the_fused_rounds_give_the_same_bits(env, n, port):
    """256-, 512- and 1024-thread workgroups of the fused-rounds kernel (tile rows of different widths, up
    to 144 KB of LDS), with the library's rows per thread and with fewer: same bits as single rounds, for
    16-byte column groups with a scalar tail and for an unaligned layout; exact averaging, fused iterations
    and the mixing rounds of the comparison topologies likewise (those against the oracle too)."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    tau = OS.num_rounds(n)
    rounds = tau + 1
    d = 4 * (37 if n > 1000 else 301) + 3
    x0 = WL.initial_state(n, d, seed=n + port)
    ref = make_state(torch, x0)
    for r in range(rounds):
        P.ceca_gossip_round(ref, ref, n, d, r % tau, port)
    x, y = OC.run(x0, port, 0.0, None, rounds, store32=True)
    gx, gy = split_state(ref, n, d)
    assert max(rel_err(gx, x)) <= 1e-5 and max(rel_err(gy, y)) <= 1e-5
    avg_ref = make_state(torch, x0)
    for r in range(tau):
        P.ceca_gossip_round(avg_ref, avg_ref, n, d, r, port)
    # an unaligned copy of the same state: rows of d + 1 floats starting 4 bytes into an allocation
    flat = torch.full((2 * n * (d + 1) + 1,), float("nan"), dtype=torch.float32, device="cuda")
    topos = {"ring": [P.ceca_topology_round(Bn.TOPO_RING, n)], "static": [P.ceca_topology_round(Bn.TOPO_STATIC_EXP, n)],
             "one_peer": [P.ceca_topology_round(Bn.TOPO_ONE_PEER_EXP, n, k) for k in range(max(tau, 1))]}
    mixed = {}
    # four iterations from round 1 with a state whose y matters, step by step
    y0 = WL.initial_state(n, d, seed=n + 77)
    cdev = torch.from_numpy(WL.quad_centers(n, d, 6)).cuda()
    steps_ref = make_state(torch, x0, y0=y0)
    for t in range(4):
        P.dsgd_ceca_step(steps_ref, steps_ref, n, d, Bn.make_quad_center_loss(cdev, 0.01, 5, 3 + t), None, 0.1,
                         (1 + t) % max(tau, 1), port)
    try:
        for threads in (256, 512, 1024):
            for rows in (0, 5):
                P.ceca_set_option(Bn.OPT_TILE_THREADS, threads)
                P.ceca_set_option(Bn.OPT_ROWS, rows)
                S = make_state(torch, x0)
                T = torch.full_like(S, float("nan"))
                P.ceca_gossip_rounds(S, T, n, d, rounds, port)
                assert torch.equal(T, ref), (threads, rows)
                U = flat[1:].view(2 * n, d + 1)
                U[:, :d] = make_state(torch, x0)
                P.ceca_gossip_rounds(U, U, n, d, rounds, port, ld=d + 1)
                assert torch.equal(U[:, :d], ref), (threads, rows, "unaligned")
                X = torch.from_numpy(x0).cuda()
                P.ceca_average(X, X, n, d, port)
                assert torch.equal(X, avg_ref[:n]), (threads, rows, "average")
                if threads == 256:
                    # the register-lean forms of the 256-thread kernel (4, 5 or 6 wavefronts per SIMD) and the plain one
                    for lean in (1, 4, 5, 6):
                        P.ceca_set_option(Bn.OPT_LEAN_TILES, lean)
                        T.fill_(float("nan"))
                        P.ceca_gossip_rounds(S, T, n, d, rounds, port)
                        assert torch.equal(T, ref), (threads, rows, "lean", lean)
                        X = torch.from_numpy(x0).cuda()
                        P.ceca_average(X, X, n, d, port)
                        assert torch.equal(X, avg_ref[:n]), (threads, rows, "average, lean", lean)
                    P.ceca_set_option(Bn.OPT_LEAN_TILES, 0)
                A = make_state(torch, x0, y0=y0)
                B = torch.full_like(A, float("nan"))
                P.dsgd_ceca_steps(A, B, n, d, Bn.make_quad_center_loss(cdev, 0.01, 5, 3), 0.1, 1 % max(tau, 1), 4, port)
                assert torch.equal(B, steps_ref), (threads, rows, "steps")
                for name, specs in topos.items():
                    X = torch.from_numpy(x0).cuda()
                    Y = torch.full_like(X, float("nan"))
                    P.ceca_mix_rounds(X, Y, n, d, specs, 3, k0=1)
                    if name not in mixed:
                        mixed[name] = Y                     # first pass: 256-thread tiles, checked against the oracle below
                    assert torch.equal(Y, mixed[name]), (threads, rows, name)
    finally:
        P.ceca_reset_options()
    otop = {"ring": [OT.ring(n)], "static": [OT.static_exponential(n)],
            "one_peer": [OT.one_peer_exponential(n, k) for k in range(max(tau, 1))]}
    for name, specs in otop.items():
        want = OT.run(x0, specs, 3, k0=1)
        assert max(rel_err(mixed[name].cpu().numpy(), want)) <= 1e-5, name


def test_long_fused_runs_on_many_agents_with_an_unaligned_layout(env):
    """More than 2048 agents, more than 16 iterations, rows that are not 16-byte aligned (scalar column
    groups, 256-thread tiles of 16 rows): same bits as single steps."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, port, steps = 3000, 9, 1, 20
    tau = OS.num_rounds(n)
    x0 = WL.initial_state(n, d, seed=12)
    cdev = torch.from_numpy(WL.quad_centers(n, d, 13)).cuda()
    A = make_state(torch, x0, ld=d + 2, offset=1)
    B = make_state(torch, x0, ld=d + 2, offset=1)
    P.dsgd_ceca_steps(A, A, n, d, Bn.make_quad_center_loss(cdev, 0.01, 2, 0), 0.1, 0, steps, port, ld=d + 2)
    for t in range(steps):
        P.dsgd_ceca_step(B, B, n, d, Bn.make_quad_center_loss(cdev, 0.01, 2, t), None, 0.1, t % tau, port, ld=d + 2)
    assert torch.equal(A[:, :d], B[:, :d])
