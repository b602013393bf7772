"""GPU parity: ceca_gossip_round through the C ABI against the fp64 oracle (mirror mode)."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as OC
from oracle import consensus as OCONS
from oracle import schedule as OS
from gpu_util import make_state, rel_err, split_state

pytestmark = pytest.mark.gpu

TOL_ROUND = 1e-5      # max relative error per gossip round
TOL_CONS = 1e-6       # consensus error after tau rounds, relative to ||mean||


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available(), "these tests need the MI355X"
    P.lib()
    return torch, P


def _run_rounds(torch, P, x0, port, rounds, ld=None, offset=0, inplace=False, y0=None):
    n, d = x0.shape
    S = make_state(torch, x0, y0=y0, ld=ld, offset=offset)
    T = S if inplace else make_state(torch, np.zeros_like(x0), ld=ld, offset=offset)
    tau = OS.num_rounds(n)
    out = []
    for k in range(rounds):
        P.ceca_gossip_round(S, T, n, d, k % tau if tau else 0, port)
        if not inplace:
            S, T = T, S
        out.append(split_state(S, n, d))
    torch.cuda.synchronize()
    return out, S


@pytest.mark.parametrize("n,port", [(2, 1), (2, 2), (3, 2), (5, 2), (6, 1), (6, 2), (7, 2), (12, 1), (12, 2),
                                    (31, 2), (30, 1), (100, 1), (100, 2), (130, 1), (257, 2)])
@pytest.mark.parametrize("d", [1000, 2051])
def test_rounds_match_oracle(env, n, port, d):
    torch, P = env
    x0 = WL.initial_state(n, d, seed=100 * n + port)
    tau = OS.num_rounds(n)
    got, _ = _run_rounds(torch, P, x0, port, tau + 1)
    x = y = x0.astype(np.float64)
    for k in range(tau + 1):
        x, y = OC.gossip_round(x, y, k % tau, port, store32=True)
        assert max(rel_err(got[k][0], x)) <= TOL_ROUND, (k, "x")
        assert max(rel_err(got[k][1], y)) <= TOL_ROUND, (k, "y")
        if k == tau - 1:
            m = OCONS.consensus_error(got[k][0])
            assert m["max_dev"] <= TOL_CONS * m["mean_norm"]
            assert np.abs(got[k][0] - x0.astype(np.float64).mean(0)).max() <= 2e-6


def test_worked_example_n6(env, golden):
    """The paper's n = 6 tables (App. B.1.1) straight through the device path; J(0) = 0."""
    torch, P = env
    for port, name in [(2, "ceca_n6_values_2p.txt"), (1, "ceca_n6_values_1p.txt")]:
        rows = {int(l.split()[0]): [float(v) for v in l.split()[1:]] for l in golden(name)}
        u = np.array(rows[0][0::2])[:, None] * np.ones((1, 8))
        got, _ = _run_rounds(torch, P, u, port, 3, y0=np.zeros_like(u))
        for r in range(3):
            assert np.allclose(got[r][0][:, 3], rows[r + 1][0::2], rtol=1e-6)
            assert np.allclose(got[r][1][:, 5], rows[r + 1][1::2], rtol=1e-6)


@pytest.mark.parametrize("n,port", [(5, 2), (6, 1), (100, 2)])
def test_layout_variants_are_bit_identical(env, n, port):
    """Padding (ld > d), an unaligned base, in-place one-port rounds and every launch shape give the
    same bits, and padding columns are never written."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    d = 1543
    x0 = WL.initial_state(n, d, seed=n)
    tau = OS.num_rounds(n)
    ref, _ = _run_rounds(torch, P, x0, port, tau)
    for ld, off in [(d + 9, 0), (d, 1), (d + 1, 3), (1544, 0)]:
        got, S = _run_rounds(torch, P, x0, port, tau, ld=ld, offset=off)
        assert np.array_equal(got[-1][0], ref[-1][0]) and np.array_equal(got[-1][1], ref[-1][1])
        if ld > d:
            assert bool((S[:, d:] == 12345.0).all())
    try:
        for seg, unr in [(1, 1), (3, 2), (7, 4), (1000, 8), (0, 2), (5, 8)]:
            P.ceca_set_option(Bn.OPT_SEGMENT, seg)
            P.ceca_set_option(Bn.OPT_ROWS, unr)
            got, _ = _run_rounds(torch, P, x0, port, tau)
            for k in range(tau):
                assert np.array_equal(got[k][0], ref[k][0]) and np.array_equal(got[k][1], ref[k][1]), (seg, unr, k)
    finally:
        P.ceca_set_option(Bn.OPT_SEGMENT, 0)
        P.ceca_set_option(Bn.OPT_ROWS, 0)
    # in place: one-port pairs and whole two-port cycles read every row before they write it
    got, _ = _run_rounds(torch, P, x0, port, tau, inplace=True)
    for k in range(tau):
        assert np.array_equal(got[k][0], ref[k][0]) and np.array_equal(got[k][1], ref[k][1])


def test_degenerate_sizes(env):
    torch, P = env
    # one agent: a round is a copy
    x0 = WL.initial_state(1, 37, seed=1)
    y0 = WL.initial_state(1, 37, seed=2)
    got, _ = _run_rounds(torch, P, x0, 2, 1, y0=y0)
    assert np.array_equal(got[0][0], x0.astype(np.float64)) and np.array_equal(got[0][1], y0.astype(np.float64))
    # one column, two agents
    x0 = np.array([[1.0], [3.0]], dtype=np.float32)
    for port in (1, 2):
        got, _ = _run_rounds(torch, P, x0, port, 1)
        assert np.array_equal(got[0][0], [[2.0], [2.0]])
        assert np.array_equal(got[0][1], [[3.0], [1.0]])      # J = mean of the others
    # round 0 never reads y: NaNs there must not leak
    x0 = WL.initial_state(6, 64, seed=3)
    got, _ = _run_rounds(torch, P, x0, 2, 3, y0=np.full((6, 64), np.nan, dtype=np.float32))
    assert np.isfinite(got[0][0]).all() and np.isfinite(got[0][1]).all()
    assert np.abs(got[2][0] - x0.astype(np.float64).mean(0)).max() < 1e-6


def test_device_call_errors(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    S = torch.zeros((12, 16), dtype=torch.float32, device="cuda")
    T = torch.zeros_like(S)
    for args, code in [((S, T, 6, 16, -1, 2), Bn.CECA_EINVAL), ((S, T, 6, 16, 3, 2), Bn.CECA_EINVAL),
                       ((S[:10], T[:10], 5, 16, 0, 1), Bn.CECA_EODD1P), ((S, T, 6, 0, 0, 2), Bn.CECA_EINVAL)]:
        with pytest.raises(P.CecaError) as e:
            P.ceca_gossip_round(*args)
        assert e.value.code == code
    # partial overlap is rejected for either port
    flat = torch.zeros(12 * 16 + 16, dtype=torch.float32, device="cuda")
    with pytest.raises(P.CecaError):
        P.ceca_gossip_round(flat[:192].view(12, 16), flat[16:208].view(12, 16), 6, 16, 0, 1)
    with pytest.raises(P.CecaError):
        P.ceca_gossip_round(flat[:192].view(12, 16), flat[16:208].view(12, 16), 6, 16, 0, 2)


@pytest.mark.parametrize("port", [1, 2])
def test_full_size_gossip_sampled_columns(env, port):
    """n = 100, d = 2^20 in the launch shape the benchmark times; the oracle follows sampled columns
    (columns are independent CECA instances), consensus is checked over everything."""
    torch, P = env
    n, d = 100, 1 << 20
    S = torch.empty((2 * n, d), dtype=torch.float32, device="cuda")
    WL.device_normal((n, d), seed=2, out=S[:n])
    S[n:] = S[:n]
    T = torch.empty_like(S)
    cols = WL.sample_columns(d, 2048, seed=2, tail=8)
    tc = torch.from_numpy(cols).cuda()
    x = y = S[:n][:, tc].cpu().numpy().astype(np.float64)
    mean_all = S[:n].double().mean(0)
    tau = OS.num_rounds(n)
    for r in range(tau):
        P.ceca_gossip_round(S, T, n, d, r, port)
        S, T = T, S
        x, y = OC.gossip_round(x, y, r, port, store32=True)
        gx, gy = S[:n][:, tc].cpu().numpy(), S[n:][:, tc].cpu().numpy()
        assert max(rel_err(gx, x)) <= TOL_ROUND and max(rel_err(gy, y)) <= TOL_ROUND, r
    dev = (S[:n].double() - mean_all).norm(dim=1).max().item()
    assert dev <= TOL_CONS * mean_all.norm().item()


@pytest.mark.parametrize("n,port", [(2, 1), (3, 2), (5, 2), (6, 1), (16, 2), (17, 2), (31, 2), (32, 1), (33, 2),
                                    (100, 1), (100, 2), (258, 1), (400, 2), (640, 1), (641, 2), (800, 2), (1023, 2),
                                    (1026, 1), (1200, 1), (1281, 2), (1500, 2), (1537, 2)])
def test_fused_rounds_equal_separate_rounds(env, n, port):
    """ceca_gossip_rounds: same bits as the sequence of single rounds, and the oracle's values."""
    torch, P = env
    d = 1037 if n < 200 else 203
    x0 = WL.initial_state(n, d, seed=7 * n + port)
    tau = OS.num_rounds(n)
    for rounds in (1, tau, tau + 1, 2 * tau + 3):
        ref, _ = _run_rounds(torch, P, x0, port, rounds)
        S = make_state(torch, x0, y0=np.full_like(x0, np.nan))      # y(0) must not be read
        T = make_state(torch, np.zeros_like(x0))
        P.ceca_gossip_rounds(S, T, n, d, rounds, port)
        gx, gy = split_state(T, n, d)
        assert np.array_equal(gx, ref[-1][0]) and np.array_equal(gy, ref[-1][1]), rounds
    x, y = OC.run(x0, port, 0.0, None, tau + 1, store32=True)
    assert max(rel_err(gx, OC.run(x0, port, 0.0, None, 2 * tau + 3, store32=True)[0])) <= TOL_ROUND
    # in place and from an unaligned, padded layout
    S = make_state(torch, x0, ld=d + 5, offset=1)
    P.ceca_gossip_rounds(S, S, n, d, tau + 1, port)
    gx, gy = split_state(S, n, d)
    assert max(rel_err(gx, x)) <= TOL_ROUND and max(rel_err(gy, y)) <= TOL_ROUND
    mean = x0.astype(np.float64).mean(0)
    assert np.abs(gx - mean).max() <= 2e-6 and np.abs(gy - mean).max() <= 2e-6
    assert bool((S[:, d:] == 12345.0).all())


def test_fused_rounds_tile_shapes_bit_identical(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d = 37, 1100
    x0 = WL.initial_state(n, d, seed=3)
    outs = []
    try:
        for rows in (0, 4, 8, 16):
            P.ceca_set_option(Bn.OPT_ROWS, rows)
            S, T = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
            P.ceca_gossip_rounds(S, T, n, d, 7, 2)
            outs.append(T.cpu().numpy())
    finally:
        P.ceca_set_option(Bn.OPT_ROWS, 0)
    assert all(np.array_equal(o, outs[0]) for o in outs[1:])


def test_fused_rounds_fallbacks(env):
    torch, P = env
    # one agent: copies; more agents than one workgroup can hold: one launch per round
    x0 = WL.initial_state(1, 33, seed=5)
    S, T = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
    P.ceca_gossip_rounds(S, T, 1, 33, 3, 2)
    assert np.array_equal(split_state(T, 1, 33)[0], x0.astype(np.float64))
    n, d = 4100, 40
    x0 = WL.initial_state(n, d, seed=6)
    tau = OS.num_rounds(n)
    for port in (1, 2):
        S, T = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
        P.ceca_gossip_rounds(S, T, n, d, tau, port)
        gx, _ = split_state(T, n, d)
        assert np.abs(gx - x0.astype(np.float64).mean(0)).max() <= 2e-6
    with pytest.raises(P.CecaError):
        P.ceca_gossip_rounds(S, T, n, d, 0, 2)


@pytest.mark.parametrize("n", [130, 1026])
@pytest.mark.parametrize("port", [1, 2])
def test_finite_time_consensus_residue(env, n, port):
    """The paper's consensus experiment (Sec. 5, finite-time exact consensus; n = 130 and n = 1026 are its
    comparison sizes): the residue sum_i ||x_i - x*|| after every round, measured on the device with
    consensus_error, follows the oracle and drops to rounding level exactly at round tau."""
    torch, P = env
    d = 256
    x0 = WL.initial_state(n, d, seed=n)
    tau = OS.num_rounds(n)
    S, T = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
    ws = torch.empty(P.consensus_error_workspace_bytes(n, d), dtype=torch.uint8, device="cuda")
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    x = y = x0.astype(np.float64)
    residues = []
    for r in range(tau):
        P.ceca_gossip_round(S, T, n, d, r, port)
        S, T = T, S
        P.consensus_error(S[:n], n, d, out, workspace=ws)
        got = out.cpu().numpy()
        x, y = OC.gossip_round(x, y, r, port, store32=True)
        want = OCONS.consensus_error(x)
        residues.append(got[1])
        if r < tau - 1:
            assert np.isclose(got[1], want["residue"], rtol=1e-5)
            assert got[1] > 1e-3 * n                      # not at consensus before the last round
    assert residues[-1] <= 1e-6 * n * np.sqrt(d) * 0.2      # ~1e-7 per entry
    assert all(b < a for a, b in zip(residues, residues[1:]))


@pytest.mark.parametrize("n,port", [(1, 2), (2, 1), (3, 2), (5, 2), (6, 1), (31, 2), (30, 1), (100, 1), (100, 2), (130, 1),
                                    (258, 1), (400, 2), (512, 1), (513, 2), (704, 1), (705, 2), (800, 2), (1023, 2), (1026, 1),
                                    (1200, 1), (1500, 2), (4096, 2)])
@pytest.mark.parametrize("d,pad,off", [(1037, 3, 0), (256, 0, 1)])
def test_exact_averaging_call(env, n, port, d, pad, off):
    """ceca_average: every output row is the plain column mean (the definition; 1e-6 relative to its
    norm), the rows are the x rows of ceca_gossip_rounds(rounds = tau) bit for bit, in place or not."""
    torch, P = env
    if n > 1000:
        d = 64 + (d % 5)
    ld = d + pad
    x0 = WL.initial_state(n, d, seed=11 * n + port)
    buf = torch.full((n * ld + off + 8,), 12345.0, dtype=torch.float32, device="cuda")
    X = buf[off: off + n * ld].view(n, ld)
    X[:, :d] = torch.from_numpy(x0).cuda()
    Y = torch.full_like(X, 12345.0)
    P.ceca_average(X, Y, n, d, port, ld=ld)
    got = Y[:, :d].cpu().numpy().astype(np.float64)
    mean = x0.astype(np.float64).mean(axis=0)
    assert np.sqrt(((got - mean) ** 2).sum(axis=1)).max() <= 1e-6 * max(np.sqrt((mean ** 2).sum()), 1e-30) + 1e-7
    assert bool((Y[:, d:] == 12345.0).all())
    tau = OS.num_rounds(n)
    if n > 1:
        S = make_state(torch, x0, y0=np.full_like(x0, np.nan))
        T = make_state(torch, np.zeros_like(x0))
        P.ceca_gossip_rounds(S, T, n, d, tau, port)
        assert np.array_equal(split_state(T, n, d)[0], got)
    P.ceca_average(X, X, n, d, port, ld=ld)
    assert torch.equal(X[:, :d], Y[:, :d])


@pytest.mark.parametrize("n,port", [(130, 2), (400, 2), (640, 1), (800, 2), (1026, 1), (1200, 2), (1500, 2)])
def test_exact_averaging_at_bench_sizes(env, n, port):
    """ceca_average and ceca_gossip_rounds on 2^27 elements, every tile of the launch (the sizes of the paper's
    consensus comparison and the agent counts where the tile shape changes): each output row is the plain
    column mean, which is the definition of what tau rounds reach (Sec. 3.1 problem statement), to 1e-6 of
    its norm; sampled columns follow the oracle round by round; the x rows of both calls have the same bits."""
    torch, P = env
    d = (1 << 27) // n // 64 * 64
    tau = OS.num_rounds(n)
    X = WL.device_normal((n, d), seed=900 + n)
    mean = X.double().mean(0)
    Y = torch.empty_like(X)
    P.ceca_average(X, Y, n, d, port)
    dev = (Y.double() - mean).norm(dim=1).max().item()
    assert dev <= TOL_CONS * mean.norm().item()
    S = torch.empty((2 * n, d), dtype=torch.float32, device="cuda")
    S[:n] = X
    S[n:] = float("nan")                                     # y(0) must not be read
    T = torch.empty_like(S)
    P.ceca_gossip_rounds(S, T, n, d, tau, port)
    assert torch.equal(T[:n], Y)
    cols = np.unique(np.concatenate([np.arange(0, 70), np.arange(d - 70, d),
                                     np.random.default_rng(n).integers(0, d, 200)]))
    ct = torch.from_numpy(cols).cuda()
    x0 = X[:, ct].cpu().numpy()
    xo, yo = OC.run(x0, port, 0.0, None, tau, store32=True)
    gx, gy = T[:n][:, ct].cpu().numpy(), T[n:][:, ct].cpu().numpy()
    assert max(rel_err(gx, xo)) <= TOL_ROUND and max(rel_err(gy, yo)) <= TOL_ROUND


def test_exact_averaging_errors(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    X = torch.zeros((5, 8), dtype=torch.float32, device="cuda")
    for n, port, code in [(5, 1, Bn.CECA_EODD1P), (4, 3, Bn.CECA_EINVAL), (0, 2, Bn.CECA_EINVAL)]:
        with pytest.raises(P.CecaError) as e:
            P.ceca_average(X, X, n, 8, port)
        assert e.value.code == code
    big = torch.zeros((4097, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.ceca_average(big, big, 4097, 4, 2)
    assert e.value.code == Bn.CECA_EINVAL
