"""GPU parity: consensus_error through the C ABI against the fp64 oracle."""
import numpy as np
import pytest

import workloads as WL
from oracle import consensus as OCONS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


def _consensus(torch, P, X, n, d, want_mean=True):
    wb = P.consensus_error_workspace_bytes(n, d)
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    xbar = torch.zeros(d, dtype=torch.float32, device="cuda") if want_mean else None
    P.consensus_error(X, n, d, out, xbar=xbar, workspace=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (xbar.cpu().numpy() if want_mean else None)


@pytest.mark.parametrize("n,d", [(1, 5), (2, 1), (5, 1000), (6, 1027), (31, 4096), (100, 3000), (1023, 4096),
                                 (3, 70001)])
def test_matches_oracle(env, n, d):
    torch, P = env
    x = WL.initial_state(n, d, seed=n + d) * 3.0 + 1.5
    X = torch.from_numpy(x).cuda()
    got, xbar = _consensus(torch, P, X, n, d)
    want = OCONS.consensus_error(x)
    assert np.isclose(got[0], want["frob2"], rtol=1e-12)
    assert np.isclose(got[1], want["residue"], rtol=1e-12)
    assert np.isclose(got[2], want["max_dev"], rtol=1e-12)
    assert np.isclose(got[3], want["mean_norm"], rtol=1e-12)
    assert got[4] == n
    assert np.allclose(xbar, want["mean"].astype(np.float32), rtol=0, atol=1e-7 * np.abs(want["mean"]).max())


def test_padding_and_unaligned(env):
    torch, P = env
    n, d, ld = 7, 515, 523
    x = WL.initial_state(n, d, seed=9)
    flat = torch.full((n * ld + 1,), 7e7, dtype=torch.float32, device="cuda")
    X = flat[1:].view(n, ld)
    X[:, :d] = torch.from_numpy(x).cuda()
    got, _ = _consensus(torch, P, X, n, d)
    want = OCONS.consensus_error(x)
    assert np.isclose(got[0], want["frob2"], rtol=1e-12) and np.isclose(got[3], want["mean_norm"], rtol=1e-12)


def test_exact_consensus_reads_zero(env):
    torch, P = env
    row = WL.initial_state(1, 2048, seed=4)
    X = torch.from_numpy(np.repeat(row, 9, axis=0)).cuda()
    got, _ = _consensus(torch, P, X, 9, 2048, want_mean=False)
    assert got[0] == 0.0 and got[1] == 0.0 and got[2] == 0.0
    assert np.isclose(got[3], np.sqrt((row.astype(np.float64) ** 2).sum()), rtol=1e-13)


def test_workspace_errors(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    X = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.consensus_error(X, 4, 64, out, workspace=None)
    assert e.value.code == Bn.CECA_EWORKSPACE
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.consensus_error(X, 4, 64, out, workspace=small)
    assert e.value.code == Bn.CECA_EWORKSPACE


def test_state_consensus_distance_of_x_and_y(env):
    """The analysis' observable ||phi||_F^2 = ||x - 1 xbar^T||_F^2 + ||y - 1 ybar^T||_F^2 (App. B.3):
    consensus_error on the x rows and on the y rows of a state, which is zero for both exactly after
    tau + 1 gossip rounds and for x only after tau."""
    torch, P = env
    from oracle import schedule as OS
    n, d = 12, 1500
    x0 = WL.initial_state(n, d, seed=12)
    S = torch.from_numpy(np.vstack([x0, x0])).cuda()
    T = torch.empty_like(S)
    tau = OS.num_rounds(n)
    P.ceca_gossip_rounds(S, T, n, d, tau, 2)
    gx, _ = _consensus(torch, P, T[:n], n, d, want_mean=False)
    gy, _ = _consensus(torch, P, T[n:], n, d, want_mean=False)
    want_y = OCONS.consensus_error((n * x0.astype(np.float64).mean(0) - x0.astype(np.float64)) / (n - 1))
    assert gx[2] <= 1e-6 * gx[3]
    assert np.isclose(gy[0], want_y["frob2"], rtol=1e-5)          # y_i = mean of the others: not at consensus yet
    P.ceca_gossip_rounds(S, T, n, d, tau + 1, 2)
    gx, _ = _consensus(torch, P, T[:n], n, d, want_mean=False)
    gy, _ = _consensus(torch, P, T[n:], n, d, want_mean=False)
    assert gx[2] <= 1e-6 * gx[3] and gy[2] <= 1e-6 * gy[3]
    assert gx[0] + gy[0] <= 1e-11 * n * gx[3] ** 2


@pytest.mark.parametrize("n,d,pad", [(1, 7, 0), (5, 1000, 0), (6, 1037, 3), (31, 40_001, 7), (258, 10, 0), (1023, 4096, 0)])
def test_state_consensus_entry_point(env, n, d, pad):
    """ceca_state_consensus on a state some gossip rounds into a run: x part, y part and ||phi||_F^2
    against the fp64 oracle on the same stored state (aligned and ragged layouts, one agent)."""
    torch, P = env
    ld = d + pad
    x0 = WL.initial_state(n, d, seed=n + 1)
    y0 = WL.initial_state(n, d, seed=n + 2)
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
    S[:n, :d] = torch.from_numpy(x0).cuda()
    S[n:, :d] = torch.from_numpy(y0).cuda()
    T = torch.zeros_like(S)
    port = 2 if n % 2 else 1
    if n > 1:
        P.ceca_gossip_round(S, T, n, d, 0, port, ld=ld)
        P.ceca_gossip_round(T, S, n, d, 1, port, ld=ld)
    ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    out = torch.full((11,), -1.0, dtype=torch.float64, device="cuda")
    P.ceca_state_consensus(S, n, d, out, workspace=ws, ld=ld)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    host = S.cpu().numpy()
    want = OCONS.state_consensus(host[:n, :d], host[n:, :d])
    for off, key in ((0, "x"), (5, "y")):
        w = want[key]
        scale = max(w["mean_norm"] ** 2 * n, w["frob2"], 1e-30)
        assert abs(got[off + 0] - w["frob2"]) <= 1e-10 * scale
        assert abs(got[off + 1] - w["residue"]) <= 1e-9 * max(w["residue"], np.sqrt(scale))
        assert abs(got[off + 2] - w["max_dev"]) <= 1e-9 * max(w["max_dev"], np.sqrt(scale))
        assert abs(got[off + 3] - w["mean_norm"]) <= 1e-10 * max(w["mean_norm"], 1e-30)
        assert got[off + 4] == n
    assert got[10] == got[0] + got[5]
    assert abs(got[10] - want["phi2"]) <= 1e-10 * max(want["phi2"], n * want["x"]["mean_norm"] ** 2)


@pytest.mark.parametrize("n,d,pad,off", [(1, 5, 0, 0), (2, 1, 0, 0), (5, 1000, 0, 0), (6, 1027, 2, 0), (31, 4096, 0, 0),
                                         (100, 3000, 8, 0), (130, 515, 0, 1), (1023, 4096, 0, 0), (1026, 37, 3, 0),
                                         (3, 70001, 3, 0), (4000, 12, 0, 0), (4096, 9, 0, 0), (5000, 8, 0, 0)])
def test_single_pass_and_two_pass_forms(env, n, d, pad, off):
    """Every form of the consensus kernels -- the library's choice, the two passes (column sums first,
    deviations second), the single pass with every agent's column tile in one workgroup, and the single
    pass with one wavefront per column strip in several shapes (rows per lane, strips per wavefront) --
    against the fp64 oracle, on aligned, padded and unaligned layouts."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    ld = d + pad
    x = WL.initial_state(n, d, seed=n + d) * 2.0 + 0.7
    buf = torch.zeros(n * ld + off + 8, dtype=torch.float32, device="cuda")
    X = buf[off: off + n * ld].view(n, ld)
    X[:, :d] = torch.from_numpy(x).cuda()
    X[:, d:] = 1e30                                         # padding must never be read
    want = OCONS.consensus_error(x)
    shapes = [(1, 0, 0), (0, 0, 0), (2, 0, 0), (3, 0, 0), (3, 32, 1), (3, 5, 3), (3, 1, 2), (3, 16, 4096), (3, 7, 1)]
    for mode, rows, strips in shapes:
        P.ceca_set_option(Bn.OPT_CONS_SINGLE_PASS, mode)
        P.ceca_set_option(Bn.OPT_ROWS, rows)
        P.ceca_set_option(Bn.OPT_CONS_STRIPS, strips)
        ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:]
        out = torch.full((5,), -1.0, dtype=torch.float64, device="cuda")
        xbar = torch.zeros(d, dtype=torch.float32, device="cuda")
        P.consensus_error(X, n, d, out, xbar=xbar, workspace=ws, ld=ld)
        torch.cuda.synchronize()
        g = out.cpu().numpy()
        what = (mode, rows, strips)
        scale = max(want["frob2"], 1e-300)
        assert abs(g[0] - want["frob2"]) <= 1e-10 * scale, what
        assert abs(g[1] - want["residue"]) <= 1e-9 * max(want["residue"], 1e-300), what
        assert abs(g[2] - want["max_dev"]) <= 1e-9 * max(want["max_dev"], 1e-300), what
        assert abs(g[3] - want["mean_norm"]) <= 1e-10 * want["mean_norm"], what
        assert g[4] == n
        assert np.abs(xbar.cpu().numpy() - want["mean"]).max() <= 1e-6 * max(np.abs(want["mean"]).max(), 1.0), what
    P.ceca_reset_options()


@pytest.mark.parametrize("n,d", [(31, 1 << 16), (100, 20_000), (6, 300_000), (512, 4100), (17, 77_777)])
def test_wavefront_strip_form_is_deterministic_and_tight(env, n, d):
    """The wavefront-strip form at rtol 1e-12 on the four scalars (as the default form is gated above), twice
    with the same bits, for layouts with and without 16-byte alignment."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    x = WL.initial_state(n, d, seed=n + d) * 3.0 + 1.5
    want = OCONS.consensus_error(x)
    for off in (0, 1):
        buf = torch.zeros(n * d + 8, dtype=torch.float32, device="cuda")
        X = buf[off: off + n * d].view(n, d)
        X.copy_(torch.from_numpy(x))
        P.ceca_set_option(Bn.OPT_CONS_SINGLE_PASS, 3)
        ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
        ws = ws[(-ws.data_ptr()) % 256:]
        outs = []
        for _ in range(2):
            ws.fill_(0xFF)                                   # stale workspace contents must not matter
            out = torch.full((5,), -1.0, dtype=torch.float64, device="cuda")
            P.consensus_error(X, n, d, out, workspace=ws)
            outs.append(out.cpu().numpy())
        assert np.array_equal(outs[0], outs[1])
        g = outs[0]
        assert np.isclose(g[0], want["frob2"], rtol=1e-12) and np.isclose(g[1], want["residue"], rtol=1e-12)
        assert np.isclose(g[2], want["max_dev"], rtol=1e-12) and np.isclose(g[3], want["mean_norm"], rtol=1e-12)
    P.ceca_reset_options()


def test_stream_probe_values(env):
    """The measurement aid computes what its header says (elementwise, in and out of place)."""
    torch, P = env
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    a = torch.randn(4096 + 8, device="cuda", generator=g)[:4096]
    b = torch.randn(4096, device="cuda", generator=g)
    c = torch.randn(4096, device="cuda", generator=g)
    o1, o2 = torch.empty_like(a), torch.empty_like(a)
    P.ceca_stream_probe(a, b, c, o1, o2, 4096)
    w1 = 0.5 * a + 0.5 * (b - 0.1 * (b - c))
    w2 = 0.4 * b + 0.6 * (a - 0.1 * (a - c))
    assert torch.allclose(o1, w1, rtol=1e-6, atol=1e-6) and torch.allclose(o2, w2, rtol=1e-6, atol=1e-6)
    a2, b2 = a.clone(), b.clone()
    P.ceca_stream_probe(a2, b2, c, a2, b2, 4096)
    assert torch.equal(a2, o1) and torch.equal(b2, o2)
    # fewer reads stand in the first array for the missing ones; fewer writes leave the other output alone
    p1, p2 = torch.full_like(a, 7.0), torch.full_like(a, 7.0)
    P.ceca_stream_probe(a, b, None, p1, p2, 4096, reads=2, writes=2)
    assert torch.allclose(p1, 0.5 * a + 0.5 * (b - 0.1 * (b - a)), rtol=1e-6, atol=1e-6)
    p1.fill_(7.0); p2.fill_(7.0)
    P.ceca_stream_probe(a, None, None, p1, None, 4096, reads=1, writes=1)
    assert torch.allclose(p1, a, rtol=1e-6, atol=1e-6) and bool((p2 == 7.0).all())
    p1.fill_(7.0)
    P.ceca_stream_probe(a, b, c, p1, None, 4096, reads=3, writes=0)
    assert bool((p1 == 7.0).all())
    with pytest.raises(P.CecaError):
        P.ceca_stream_probe(a, b, c, o1, o2, 4095)
    with pytest.raises(P.CecaError):
        P.ceca_stream_probe(a, b, c, o1, o2, 4096, reads=4)
