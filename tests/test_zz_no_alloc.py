"""GPU: consensus_error_noalloc (the entry point for callers that cannot allocate device memory) through
the C ABI against consensus_error with a caller workspace -- same kernels, same launch shapes, so the five
results are the same doubles -- and against the fp64 oracle, on two calls in a row of which the second has
the smaller input (the library's scratch array keeps the first call's contents).

Collected last on purpose (file name): the round's end stops at the first failing test."""
import ctypes

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


def _with_workspace(torch, P, X, n, d, ld):
    ws = torch.empty(P.consensus_error_workspace_bytes(n, d) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    out = torch.full((5,), -1.0, dtype=torch.float64, device="cuda")
    xbar = torch.full((d,), -1.0, dtype=torch.float32, device="cuda")
    P.consensus_error(X, n, d, out, xbar=xbar, workspace=ws, ld=ld)
    torch.cuda.synchronize()
    return out.cpu().numpy(), xbar.cpu().numpy()


def _noalloc(torch, P, X, n, d, ld):
    """Straight through the C ABI: plain pointers and sizes, the stream torch is on."""
    L = P.lib()
    out = torch.full((5,), -2.0, dtype=torch.float64, device="cuda")
    xbar = torch.full((d,), -2.0, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rc = L.consensus_error_noalloc(ctypes.c_void_p(X.data_ptr()), n, d, ld, ctypes.c_void_p(out.data_ptr()),
                                   ctypes.c_void_p(xbar.data_ptr()), ctypes.c_void_p(stream) if stream else None)
    assert rc == 0, L.ceca_last_error().decode()
    torch.cuda.synchronize()
    return out.cpu().numpy(), xbar.cpu().numpy()


def _check(got, xbar, ref, ref_xbar, x):
    want = OCONS.consensus_error(x)
    assert np.array_equal(got, ref), (got, ref)                 # same kernels and launch shapes: same doubles
    assert np.array_equal(xbar, ref_xbar)
    assert np.isclose(got[0], want["frob2"], rtol=1e-12) and np.isclose(got[1], want["residue"], rtol=1e-12)
    assert np.isclose(got[2], want["max_dev"], rtol=1e-12) and np.isclose(got[3], want["mean_norm"], rtol=1e-12)
    assert got[4] == x.shape[0]
    assert np.abs(xbar - want["mean"]).max() <= 1e-6 * max(np.abs(want["mean"]).max(), 1.0)


# (first call, second and smaller call, form): every form of the kernels -- the library's choice (wavefront
# strips up to 512 agents, workgroup tiles or two passes beyond), and the two passes forced -- ragged and
# padded layouts included
@pytest.mark.parametrize("first,second,form", [((31, 300_007, 300_007 + 9), (31, 4099, 4099), 1),
                                               ((100, 65_536, 65_536), (6, 1000, 1000), 1),
                                               ((1023, 4096, 4096), (130, 515, 520), 1),
                                               ((5000, 64, 64), (5, 1000, 1000), 1),
                                               ((40, 50_000, 50_000), (7, 3001, 3001), 0),
                                               ((200, 8192, 8192), (31, 4096, 4096), 2)])
def test_two_calls_in_a_row_match_the_workspace_entry_point(env, first, second, form):
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    P.ceca_set_option(Bn.OPT_CONS_SINGLE_PASS, form)          # (undone after the test by the suite's fixture)
    for n, d, ld in (first, second):
        x = WL.initial_state(n, d, seed=n + d) * 2.0 + 0.7
        X = torch.full((n, ld), 1e30, dtype=torch.float32, device="cuda")      # padding must never be read
        X[:, :d] = torch.from_numpy(x).cuda()
        ref, ref_xbar = _with_workspace(torch, P, X, n, d, ld)
        got, xbar = _noalloc(torch, P, X, n, d, ld)
        _check(got, xbar, ref, ref_xbar, x)


def test_binding_and_null_mean(env):
    torch, P = env
    n, d = 12, 2051
    x = WL.initial_state(n, d, seed=5)
    X = torch.from_numpy(x).cuda()
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    P.consensus_error_noalloc(X, n, d, out)                  # no mean asked for
    torch.cuda.synchronize()
    ref, _ = _with_workspace(torch, P, X, n, d, d)
    assert np.array_equal(out.cpu().numpy(), ref)


def test_sizes_beyond_the_scratch_array_are_refused(env):
    """A problem whose partial sums exceed the 16 MiB array returns CECA_EWORKSPACE and launches nothing;
    the next call works."""
    torch, P = env
    from paper_2306_00256_amd import binding as Bn
    n, d = 8, 3_000_000                                      # two-pass form (forced): d fp64 column sums = 24 MB
    X = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    out = torch.full((5,), -3.0, dtype=torch.float64, device="cuda")
    P.ceca_set_option(Bn.OPT_CONS_SINGLE_PASS, 0)
    try:
        with pytest.raises(P.CecaError) as e:
            P.consensus_error_noalloc(X, n, d, out)
        assert e.value.code == Bn.CECA_EWORKSPACE and "16777216" in str(e.value)
    finally:
        P.ceca_reset_options()
    torch.cuda.synchronize()
    assert bool((out == -3.0).all())
    with pytest.raises(P.CecaError):
        P.consensus_error_noalloc(X, 0, d, out)
    P.consensus_error_noalloc(X, n, d, out)                  # the library's own form fits
    torch.cuda.synchronize()
    assert out.cpu().numpy()[4] == n
