"""GPU parity: dsgd_ceca_run (several minibatch iterations per call; each iteration after the first finishes
the iteration before inside its gradient kernel: one kernel per iteration where the one-pass gradient
applies, two where the gradient takes two passes) against single dsgd_ceca_step calls (bit for bit) and
against the fp64 oracle (1e-4 over the run)."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as OC
from oracle import losses as OL
from oracle import schedule as OS
from gpu_util import make_state, rel_err, split_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


def _aligned(torch, nbytes):
    buf = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    return buf[(-buf.data_ptr()) % 256:][:nbytes]


def _problem(torch, Bn, kind, n, N, d, B, iters, seed, noise=0.0):
    if kind == "lsq":
        A, t, _ = WL.lsq_data(n, N, d, seed=seed)
    else:
        A, t, _ = WL.logistic_data_sparse(n, N, d, seed=seed, density=0.5)
    idx = WL.batch_indices(n, N, B, iters, seed=seed)
    Ad, td, idxd = torch.from_numpy(A).cuda(), torch.from_numpy(t).cuda(), torch.from_numpy(idx).cuda()
    code = Bn.LOSS_LSQ if kind == "lsq" else Bn.LOSS_LOGISTIC
    return A, t, idx, Ad, td, idxd, code


@pytest.mark.parametrize("kind", ["lsq", "logistic"])
@pytest.mark.parametrize("n,port,d,B,ld", [(130, 2, 4096, 16, None), (128, 1, 2052, 5, 2056), (129, 2, 8192, 9, None),
                                           (130, 1, 16384, 3, None), (131, 2, 1100, 40, None),
                                           (6, 1, 1000, 8, None), (5, 2, 4100, 7, None), (130, 2, 515, 4, None),
                                           (258, 1, 10, 50, None), (12, 2, 63, 9, None), (9, 2, 255, 20, 258),
                                           (6, 1, 1023, 12, None), (6, 2, 1027, 5, None), (4, 2, 1000, 40, None),
                                           (6, 2, 10000, 32, None), (30, 1, 8192, 16, 8192 + 64), (7, 2, 2000, 33, 2064),
                                           (6, 1, 1500, 6, 1501)])
def test_run_equals_single_steps_and_oracle(env, kind, n, port, d, B, ld):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    N, iters, k0, lr, noise = 10, 7, 4, 0.002, 0.05
    A, t, idx, Ad, td, idxd, code = _problem(torch, Bn, kind, n, N, d, B, iters, seed=n + d)
    tau = OS.num_rounds(n)
    x0 = 0.05 * WL.initial_state(n, d, seed=n + 1)
    y0 = 0.05 * WL.initial_state(n, d, seed=n + 2)
    mk = lambda k: Bn.make_minibatch_loss(code, Ad, td, N, B, noise_std=noise, seed=9, k=k)
    # reference: one dsgd_ceca_step per iteration
    ws1 = _aligned(torch, P.dsgd_ceca_workspace_bytes(n, d, mk(0)))
    S = make_state(torch, x0, y0=y0, ld=ld)
    T = S if port == 1 else make_state(torch, np.zeros_like(x0), ld=ld)
    mid = None
    for t_ in range(iters):
        if t_ == iters - 1:
            mid = S.clone()                                  # the state after iters - 1 iterations
        P.dsgd_ceca_step(S, T, n, d, mk(k0 + t_), idxd[t_], lr, (k0 + t_) % tau, port, workspace=ws1)
        if T is not S:
            S, T = T, S
    rx, ry = split_state(S, n, d)
    ws = _aligned(torch, P.dsgd_ceca_run_workspace_bytes(n, d, mk(0)))
    # fused iterations keep the state in half-step form between them (default) or as full states with two
    # message buffers; shapes on the two-pass gradient are not affected by the switch
    for half in (1, 0):
        P.ceca_set_option(Bn.OPT_HALF_STEP_RUN, half)
        for inplace in (False, True):
            for count in (iters, iters - 1):                 # odd and even: the closing combine always reads the copy
                A_ = make_state(torch, x0, y0=y0, ld=ld)
                B_ = A_ if inplace else make_state(torch, np.zeros_like(x0), ld=ld)
                P.dsgd_ceca_run(A_, B_, n, d, mk(k0), idxd, lr, k0 % tau, count, port, workspace=ws)
                if count == iters:
                    gx, gy = split_state(B_, n, d)
                    assert np.array_equal(gx, rx) and np.array_equal(gy, ry), (half, inplace)
                else:
                    assert torch.equal(B_[:, :d], mid[:, :d]), (half, inplace, "one iteration fewer")
                if not inplace:
                    ax, ay = split_state(A_, n, d)
                    assert np.array_equal(ax, x0.astype(np.float64)) and np.array_equal(ay, y0.astype(np.float64))
                if ld is not None:
                    assert bool((B_[:, d:] == 12345.0).all())
    P.ceca_reset_options()
    grad = OL.make_minibatch_grad(kind, A, t, idx, k0=k0, noise_std=noise, seed=9)
    x, y = OC.run(x0, port, lr, grad, iters, store32=True, y0=y0, k0=k0)
    assert max(rel_err(rx, x)) <= 1e-4 and max(rel_err(ry, y)) <= 1e-4


def test_single_iteration_and_argument_errors(env):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d, N, B = 130, 4096, 6, 4
    A, t, idx, Ad, td, idxd, code = _problem(torch, Bn, "lsq", n, N, d, B, 2, seed=1)
    loss = Bn.make_minibatch_loss(code, Ad, td, N, B)
    x0 = 0.05 * WL.initial_state(n, d, seed=2)
    ws = _aligned(torch, P.dsgd_ceca_run_workspace_bytes(n, d, loss))
    S1, T1 = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
    P.dsgd_ceca_step(S1, T1, n, d, loss, idxd[0], 0.01, 0, 2, workspace=_aligned(torch, P.dsgd_ceca_workspace_bytes(n, d, loss)))
    S2, T2 = make_state(torch, x0), make_state(torch, np.zeros_like(x0))
    P.dsgd_ceca_run(S2, T2, n, d, loss, idxd, 0.01, 0, 1, 2, workspace=ws)
    assert torch.equal(T1, T2)
    for kwargs, code_ in [(dict(iters=0), Bn.CECA_EINVAL), (dict(ws=ws[:1024]), Bn.CECA_EWORKSPACE), (dict(ws=None), Bn.CECA_EWORKSPACE)]:
        with pytest.raises(P.CecaError) as e:
            P.dsgd_ceca_run(S2, T2, n, d, loss, idxd, 0.01, 0, kwargs.get("iters", 2), 2, workspace=kwargs.get("ws", ws))
        assert e.value.code == code_
    c = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    with pytest.raises(P.CecaError) as e:
        P.dsgd_ceca_run(S2, T2, n, d, Bn.make_quad_center_loss(c, 0.0, 0, 0), idxd, 0.01, 0, 2, 2, workspace=ws)
    assert e.value.code == Bn.CECA_EINVAL


@pytest.mark.parametrize("iters", [2, 3, 4, 5])
@pytest.mark.parametrize("n,port,d,B", [(6, 2, 10000, 32), (6, 1, 2051, 9)])
def test_two_pass_shapes_for_every_parity_of_the_iteration_count(env, iters, n, port, d, B):
    """Shapes on the two-pass gradient alternate the state between S_out and a copy in the workspace: the
    result must land in S_out for odd and even iteration counts, in place and out of place."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    N, lr = 12, 0.003
    A, t, idx, Ad, td, idxd, code = _problem(torch, Bn, "logistic", n, N, d, B, iters, seed=iters)
    tau = OS.num_rounds(n)
    x0 = 0.05 * WL.initial_state(n, d, seed=3)
    loss = Bn.make_minibatch_loss(code, Ad, td, N, B)
    ws1 = _aligned(torch, P.dsgd_ceca_workspace_bytes(n, d, loss))
    S = make_state(torch, x0)
    for t_ in range(iters):
        P.dsgd_ceca_step(S, S, n, d, loss, idxd[t_], lr, (1 + t_) % tau, port, workspace=ws1)
    ws = _aligned(torch, P.dsgd_ceca_run_workspace_bytes(n, d, loss))
    for inplace in (False, True):
        A_ = make_state(torch, x0)
        B_ = A_ if inplace else torch.full_like(A_, float("nan"))
        P.dsgd_ceca_run(A_, B_, n, d, loss, idxd, lr, 1 % tau, iters, port, workspace=ws)
        assert torch.equal(B_, S), (iters, inplace)
