"""GPU parity: ceca_graph_rounds (gossip over arbitrary graphs given as neighbour tables) against the
general-graph oracle, and against the shift-invariant kernel where the graph is circulant."""
import numpy as np
import pytest

import workloads as WL
from oracle import graphs as OG
from oracle import topologies as OT
from gpu_util import rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


def _dev(torch, tables):
    """Stack per-round (nbr, w, w_self) host tables of equal width into device arrays."""
    nbr = torch.from_numpy(np.stack([t[0] for t in tables]).astype(np.int32)).cuda().contiguous()
    w = torch.from_numpy(np.stack([t[1] for t in tables]).astype(np.float32)).cuda().contiguous()
    ws = torch.from_numpy(np.stack([t[2] for t in tables]).astype(np.float32)).cuda().contiguous()
    return nbr, w, ws


CASES = [("hypercube", 64, 0), ("hypercube", 1024, 0), ("torus", 15, 3), ("torus", 130, 10), ("grid", 12, 4),
         ("grid", 1026, 27), ("random", 50, 0), ("random", 700, 0), ("random", 2050, 0), ("random", 2049, 0),
         ("ring", 31, 0), ("ring", 3001, 0)]


@pytest.mark.parametrize("kind,n,rows", CASES)
def test_graph_rounds_match_the_oracle(env, kind, n, rows):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    d = (4 * 9 + 3) if n > 1000 else (4 * 150 + 3)           # 16-byte groups and a scalar tail
    rounds = 5
    edges = WL.edges_of(kind, n, rows)
    host = WL.graph_table(n, edges)
    nbr, w, ws = _dev(torch, [host])
    x0 = WL.initial_state(n, d, seed=n)
    want = OG.run(x0, [OG.metropolis(n, edges)], rounds, store32=True)
    outs = []
    try:
        for threads in (0, 256, 512, 1024):
            P.ceca_set_option(Bn.OPT_TILE_THREADS, threads)
            X = torch.from_numpy(x0).cuda()
            Y = torch.full_like(X, float("nan"))
            P.ceca_graph_rounds(X, Y, n, d, nbr, w, ws, rounds)
            outs.append(Y)
            P.ceca_graph_rounds(X, X, n, d, nbr, w, ws, rounds)                  # in place
            assert torch.equal(X, Y), threads
    finally:
        P.ceca_set_option(Bn.OPT_TILE_THREADS, 0)
    assert all(torch.equal(outs[0], o) for o in outs[1:])
    try:
        P.ceca_set_option(Bn.OPT_GRAPH_STAGE, 0)                                 # tables read from memory, not staged in LDS
        X = torch.from_numpy(x0).cuda()
        P.ceca_graph_rounds(X, X, n, d, nbr, w, ws, rounds)
        assert torch.equal(X, outs[0])
    finally:
        P.ceca_set_option(Bn.OPT_GRAPH_STAGE, 1)
    assert max(rel_err(outs[0].cpu().numpy(), want)) <= 1e-5
    # the mean of every column is kept (W is doubly stochastic)
    assert np.abs(outs[0].cpu().numpy().astype(np.float64).mean(axis=0) - x0.astype(np.float64).mean(axis=0)).max() <= 1e-6
    # unaligned layout: rows of d + 1 floats starting 4 bytes into an allocation
    flat = torch.full((n * (d + 1) + 1,), float("nan"), dtype=torch.float32, device="cuda")
    U = flat[1:].view(n, d + 1)
    U[:, :d] = torch.from_numpy(x0).cuda()
    P.ceca_graph_rounds(U, U, n, d, nbr, w, ws, rounds, ld=d + 1)
    assert torch.equal(U[:, :d], outs[0])


@pytest.mark.parametrize("n", [6, 31, 130, 1026])
def test_circulant_graphs_give_the_bits_of_the_mixing_kernel(env, n):
    """Ring, static exponential and one-peer exponential written as neighbour tables (same order of the
    neighbours, same float weights): bit-identical to ceca_mix_rounds."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    d = 4 * 60 + 2
    tau = max(OT.num_rounds(n), 1)
    x0 = WL.initial_state(n, d, seed=n + 3)
    kinds = {"ring": [P.ceca_topology_round(Bn.TOPO_RING, n)], "static": [P.ceca_topology_round(Bn.TOPO_STATIC_EXP, n)],
             "one_peer": [P.ceca_topology_round(Bn.TOPO_ONE_PEER_EXP, n, k) for k in range(tau)]}
    for name, specs in kinds.items():
        width = max(max(sp.m for sp in specs), 1)
        tables = []
        for sp in specs:
            nbr = np.tile(np.arange(n, dtype=np.int32)[:, None], (1, width))
            w = np.zeros((n, width), dtype=np.float32)
            for j in range(sp.m):
                nbr[:, j] = (np.arange(n) - sp.shift[j]) % n
                w[:, j] = sp.w[j]
            tables.append((nbr, w, np.full(n, sp.w_self, dtype=np.float32)))
        tn, tw, ts = _dev(torch, tables)
        X = torch.from_numpy(x0).cuda()
        Y = X.clone()
        P.ceca_mix_rounds(X, X, n, d, specs, 2 * tau + 1, k0=1)
        P.ceca_graph_rounds(Y, Y, n, d, tn, tw, ts, 2 * tau + 1, k0=1)
        assert torch.equal(X, Y), name


@pytest.mark.parametrize("tau", [1, 3, 6, 10])
def test_one_peer_hypercube_reaches_the_exact_mean(env, tau):
    torch, P = env
    n, d = 1 << tau, 257
    x0 = WL.initial_state(n, d, seed=tau)
    tables = []
    for k in range(tau):
        nbr = (np.arange(n, dtype=np.int32) ^ (1 << k))[:, None]
        tables.append((nbr, np.full((n, 1), 0.5, dtype=np.float32), np.full(n, 0.5, dtype=np.float32)))
    tn, tw, ts = _dev(torch, tables)
    X = torch.from_numpy(x0).cuda()
    P.ceca_graph_rounds(X, X, n, d, tn, tw, ts, tau)
    got = X.cpu().numpy()
    mean = x0.astype(np.float64).mean(axis=0)
    assert np.abs(got - mean).max() <= 1e-6
    want = OG.run(x0, [OG.one_peer_hypercube(tau, k) for k in range(tau)], tau, store32=True)
    assert max(rel_err(got, want)) <= 1e-6


def test_indices_outside_the_graph_are_clamped_and_errors(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d = 5, 64
    x0 = WL.initial_state(n, d, seed=1)
    nbr = np.array([[-7], [1], [2], [3], [99]], dtype=np.int32)          # vertex 0 reads vertex 0, vertex 4 reads vertex 4
    w = np.full((n, 1), 0.25, dtype=np.float32)
    ws = np.full(n, 0.75, dtype=np.float32)
    tn, tw, ts = _dev(torch, [(nbr, w, ws)])
    X = torch.from_numpy(x0).cuda()
    P.ceca_graph_rounds(X, X, n, d, tn, tw, ts, 1)
    clamped = np.array([[0], [1], [2], [3], [4]], dtype=np.int64)
    want = OG.run(x0, [(clamped, w.astype(np.float64), ws.astype(np.float64))], 1, store32=True)
    assert max(rel_err(X.cpu().numpy(), want)) <= 1e-6
    bad = [dict(n=0), dict(n=4097), dict(rounds=0), dict(k0=-1)]
    for kw in bad:
        with pytest.raises(P.CecaError) as e:
            P.ceca_graph_rounds(X, X, kw.get("n", n), d, tn, tw, ts, kw.get("rounds", 1), k0=kw.get("k0", 0))
        assert e.value.code == Bn.CECA_EINVAL
    with pytest.raises(P.CecaError):
        P.ceca_graph_rounds(X, X, n, d, tn, tw, None, 1)
    with pytest.raises(P.CecaError):                                      # partial overlap of input and output
        flat = torch.zeros(2 * n * d, device="cuda")
        P.ceca_graph_rounds(flat[: n * d].view(n, d), flat[d: d + n * d].view(n, d), n, d, tn, tw, ts, 1)
