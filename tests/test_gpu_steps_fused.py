"""GPU parity: dsgd_ceca_steps (several iterations with the quadratic-centre loss fused into one pass)
against single dsgd_ceca_step calls (bit for bit) and against the fp64 oracle (1e-4 over a run)."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as OC
from oracle import losses as OL
from oracle import schedule as OS
from gpu_util import make_state, rel_err, split_state

pytestmark = pytest.mark.gpu

TOL_RUN = 1e-4


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


def _single_steps(P, Bn, S, T, n, d, c, std, seed, lr, k0, steps, port):
    tau = OS.num_rounds(n)
    for k in range(k0, k0 + steps):
        P.dsgd_ceca_step(S, T, n, d, Bn.make_quad_center_loss(c, std, seed, k), None, lr, k % tau if tau else 0, port)
        if T is not S:
            S, T = T, S
    return S


@pytest.mark.parametrize("n,port", [(1, 2), (2, 2), (5, 2), (6, 1), (6, 2), (31, 2), (30, 1), (100, 2), (258, 1), (1023, 2)])
@pytest.mark.parametrize("d,ld,off", [(2051, 2051, 0), (1024, 1028, 0), (515, 515, 1)])
def test_fused_iterations_equal_single_steps_and_oracle(env, n, port, d, ld, off):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    if n > 200:
        d, ld = d // 8 + (d % 4), d // 8 + (d % 4) + (ld - d)
    seed, lr, std = 7, 0.1, 0.01
    tau = OS.num_rounds(n)
    k0, steps = 3, 2 * max(tau, 1) + 1
    c = WL.quad_centers(n, d, seed)
    x0 = WL.initial_state(n, d, seed, kind="normal")
    y0 = WL.initial_state(n, d, seed + 1, kind="normal")
    cdev = torch.from_numpy(c).cuda()
    # reference: one call per iteration
    S = make_state(torch, x0, y0=y0, ld=ld, offset=off)
    T = S if port == 1 else make_state(torch, np.zeros_like(x0), ld=ld, offset=off)
    ref = _single_steps(P, Bn, S, T, n, d, cdev, std, seed, lr, k0, steps, port)
    rx, ry = split_state(ref, n, d)
    # fused, out of place and in place
    for inplace in (False, True):
        A = make_state(torch, x0, y0=y0, ld=ld, offset=off)
        B = A if inplace else make_state(torch, np.zeros_like(x0), ld=ld, offset=off)
        P.dsgd_ceca_steps(A, B, n, d, Bn.make_quad_center_loss(cdev, std, seed, k0), lr, k0 % tau if tau else 0, steps, port)
        gx, gy = split_state(B, n, d)
        assert np.array_equal(gx, rx) and np.array_equal(gy, ry), inplace
        if ld > d:
            assert bool((B[:, d:] == 12345.0).all())
    grad = OL.make_quad_center_grad(c, std, seed)
    x, y = OC.run(x0, port, lr, grad, steps, store32=True, y0=y0, k0=k0)
    assert max(rel_err(rx, x)) <= TOL_RUN and max(rel_err(ry, y)) <= TOL_RUN


def test_first_round_zero_does_not_read_y(env):
    """Starting at round 0 (b = 0) the fused call must not let y(0) through, NaNs included."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, port = 31, 1000, 2
    c = torch.from_numpy(WL.quad_centers(n, d, 1)).cuda()
    x0 = WL.initial_state(n, d, 1)
    A = make_state(torch, x0, y0=np.full_like(x0, np.nan))
    B = make_state(torch, np.zeros_like(x0))
    P.dsgd_ceca_steps(A, B, n, d, Bn.make_quad_center_loss(c, 0.01, 1, 0), 0.1, 0, 7, port)
    assert bool(torch.isfinite(B[:, :d]).all())


def test_tile_shapes_and_long_runs(env):
    """Rows per thread do not change the bits; more iterations than one kernel takes run as several
    kernels with the same result as shorter calls and as single steps, in place and out of place."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, port, seed = 30, 1540, 1, 2
    c = torch.from_numpy(WL.quad_centers(n, d, seed)).cuda()
    x0 = WL.initial_state(n, d, seed)
    outs = []
    try:
        for rows in (0, 1, 2, 4, 8, 12, 16):
            P.ceca_set_option(Bn.OPT_ROWS, rows)
            A = make_state(torch, x0)
            P.dsgd_ceca_steps(A, A, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 0), 0.1, 0, 11, port)
            outs.append(A)
    finally:
        P.ceca_set_option(Bn.OPT_ROWS, 0)
    assert all(torch.equal(outs[0], o) for o in outs[1:])
    A = make_state(torch, x0)
    P.dsgd_ceca_steps(A, A, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 0), 0.1, 0, 70, port)     # > 64: two kernels
    Bs = make_state(torch, x0)
    P.dsgd_ceca_steps(Bs, Bs, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 0), 0.1, 0, 35, port)
    P.dsgd_ceca_steps(Bs, Bs, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 35), 0.1, 35 % 5, 35, port)
    assert torch.equal(A, Bs)
    # out of place from round 2 of the cycle, 150 iterations (three kernels), against single steps
    src = make_state(torch, x0)
    keep = src.clone()
    dst = torch.full_like(src, float("nan"))
    P.dsgd_ceca_steps(src, dst, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 7), 0.1, 2, 150, port)
    assert torch.equal(src, keep)
    R = make_state(torch, x0)
    for t in range(150):
        P.dsgd_ceca_step(R, R, n, d, Bn.make_quad_center_loss(c, 0.01, seed, 7 + t), None, 0.1, (2 + t) % 5, port)
    assert torch.equal(dst, R)


def test_rejects_other_losses(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d = 4, 64
    S = torch.zeros((2 * n, d), dtype=torch.float32, device="cuda")
    A = torch.zeros((n, 8, d), dtype=torch.float32, device="cuda")
    t = torch.zeros((n, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.dsgd_ceca_steps(S, S, n, d, Bn.make_minibatch_loss(Bn.LOSS_LSQ, A, t, 8, 4), 0.1, 0, 2, 2)
    assert e.value.code == Bn.CECA_EINVAL


@pytest.mark.parametrize("name", ["quad31_2p", "quad30_1p"])
def test_full_size_fused_run_on_sampled_columns(env, name):
    """The large workload at its full size, all 50 iterations in one fused call in the benchmark's layout;
    the oracle follows sampled columns (each column is an independent instance of the recursion)."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    sp = WL.SPECS[name]
    n, d, port = sp.n, sp.d, sp.port
    ld = (d + 63) // 64 * 64
    c = torch.empty((n, ld), dtype=torch.float32, device="cuda")
    WL.device_normal((n, ld), seed=sp.seed, out=c)
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
    T = S if port == 1 else torch.empty_like(S)
    cols = WL.sample_columns(d, 1536, seed=sp.seed, tail=8)
    tc = torch.from_numpy(cols).cuda()
    grad = OL.make_quad_center_grad(c[:, tc].cpu().numpy(), sp.noise_std, sp.seed, columns=cols)
    P.dsgd_ceca_steps(S, T, n, d, Bn.make_quad_center_loss(c, sp.noise_std, sp.seed, 0), sp.lr, 0, sp.iters, port, ld=ld)
    x, y = OC.run(np.zeros((n, len(cols))), port, sp.lr, grad, sp.iters, store32=True)
    gx, gy = T[:n][:, tc].cpu().numpy(), T[n:][:, tc].cpu().numpy()
    assert max(rel_err(gx, x)) <= TOL_RUN and max(rel_err(gy, y)) <= TOL_RUN
    xbar = T[:n, :d].double().mean(0)
    cbar = c[:, :d].double().mean(0)
    assert (xbar - cbar * (1 - (1 - sp.lr) ** sp.iters)).abs().max().item() < 0.02
