"""GPU: a run resumed from a checkpoint of (x, y, k) continues with the same bits, and the resumed
run still follows the oracle (Algorithm 1's state is exactly (x, y, k); noise is keyed by k)."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as OC
from oracle import losses as OL
from oracle import schedule as OS
from gpu_util import rel_err, split_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2306_00256_amd as P
    assert torch.cuda.is_available()
    P.lib()
    return torch, P


def _steps(P, Bn, S, T, n, d, ld, c, k0, k1, port, seed):
    tau = OS.num_rounds(n)
    for k in range(k0, k1):
        P.dsgd_ceca_step(S, T, n, d, Bn.make_quad_center_loss(c, 0.01, seed, k), None, 0.1, k % tau, port, ld=ld)
        if T is not S:
            S, T = T, S
    return S, T


@pytest.mark.parametrize("n,port", [(31, 2), (30, 1), (6, 2)])
def test_resume_is_bit_identical(env, tmp_path, n, port):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    from paper_2306_00256_amd import checkpoint as CK
    d, ld, seed, k_mid, k_end = 5003, 5056, 3, 7, 16
    c_host = WL.quad_centers(n, d, seed)
    c = torch.from_numpy(c_host).cuda()
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device="cuda")
    T = S if port == 1 else torch.zeros_like(S)
    S, T = _steps(P, Bn, S, T, n, d, ld, c, 0, k_mid, port, seed)
    path = str(tmp_path / "run.ckpt")
    CK.save_state(path, S, n, d, k_mid, meta={"port": port})
    S, T = _steps(P, Bn, S, T, n, d, ld, c, k_mid, k_end, port, seed)
    straight = split_state(S, n, d)

    R, n2, d2, k2, meta = CK.load_state(path, device="cuda", ld=d + 1)     # other (ragged) row pitch
    assert (n2, d2, k2, meta["port"]) == (n, d, k_mid, port)
    Q = R if port == 1 else torch.zeros_like(R)
    R, Q = _steps(P, Bn, R, Q, n, d, d + 1, c, k2, k_end, port, seed)
    resumed = split_state(R, n, d)
    assert np.array_equal(straight[0], resumed[0]) and np.array_equal(straight[1], resumed[1])

    grad = OL.make_quad_center_grad(c_host, 0.01, seed)
    x, y = OC.run(np.zeros((n, d)), port, 0.1, grad, k_end, store32=True)
    assert max(rel_err(resumed[0], x)) <= 1e-4 and max(rel_err(resumed[1], y)) <= 1e-4
