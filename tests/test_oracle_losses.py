"""Pins for oracle/losses.py, oracle/noise.py, oracle/consensus.py (CPU only): finite differences,
closed forms, distribution checks, the noise-free quadratic trajectory."""
import numpy as np
import pytest

import workloads as WL
from oracle import ceca as C
from oracle import consensus, losses, noise
from oracle import schedule as S


def _fd(f, z, h=1e-6):
    g = np.zeros_like(z)
    for j in range(z.size):
        zp, zm = z.copy(), z.copy()
        zp[j] += h
        zm[j] -= h
        g[j] = (f(zp) - f(zm)) / (2 * h)
    return g


@pytest.mark.parametrize("fn", [losses.lsq_loss_and_grad, losses.logistic_loss_and_grad])
def test_gradients_match_finite_differences(fn):
    rng = np.random.default_rng(3)
    Ab = rng.standard_normal((5, 7))
    t = rng.standard_normal(5) if fn is losses.lsq_loss_and_grad else np.sign(rng.standard_normal(5))
    z = rng.standard_normal(7)
    g = fn(Ab, t, z)[1]
    assert np.allclose(g, _fd(lambda w: fn(Ab, t, w)[0], z), rtol=1e-6, atol=1e-8)


def test_single_row_closed_forms():
    a = np.array([[1.0, -2.0, 0.5]])
    z = np.array([0.3, 0.1, -0.4])
    # least squares, B = 1: (a.z - t) a
    assert np.allclose(losses.lsq_loss_and_grad(a, np.array([2.0]), z)[1], (a[0] @ z - 2.0) * a[0])
    # logistic, B = 1, y = -1: sigma(a.z) a
    s = 1.0 / (1.0 + np.exp(-(a[0] @ z)))
    assert np.allclose(losses.logistic_loss_and_grad(a, np.array([-1.0]), z)[1], s * a[0])
    # and y = +1: -(1 - sigma(a.z)) a
    assert np.allclose(losses.logistic_loss_and_grad(a, np.array([1.0]), z)[1], -(1 - s) * a[0])


def test_lsq_gradient_vanishes_at_noiseless_solution():
    A, b, xs = WL.lsq_data(3, 16, 20, seed=5, obs_noise=0.0)
    idx = WL.batch_indices(3, 16, 4, 2, seed=5)
    g = losses.make_minibatch_grad("lsq", A, b, idx)
    z = np.tile(xs.astype(np.float64), (3, 1))
    assert np.abs(g(z, 0)).max() < 1e-4        # b was rounded to fp32


def test_logistic_large_margin_is_stable():
    a = np.array([[1000.0]])
    for y in (-1.0, 1.0):
        l, g = losses.logistic_loss_and_grad(a, np.array([y]), np.array([1.0]))
        assert np.isfinite(l) and np.isfinite(g).all()


def test_minibatch_uses_the_agents_own_rows():
    A, b, _ = WL.lsq_data(4, 8, 6, seed=1)
    idx = WL.batch_indices(4, 8, 3, 5, seed=1)
    g = losses.make_minibatch_grad("lsq", A, b, idx)
    z = np.random.default_rng(0).standard_normal((4, 6))
    e = g(z, 2)
    for i in range(4):
        rows = idx[2, i]
        ref = sum((A[i, j].astype(float) @ z[i] - float(b[i, j])) * A[i, j].astype(float) for j in rows) / 3
        assert np.allclose(e[i], ref)


def test_noise_distribution():
    cols = np.arange(400_000)
    e = noise.normals(3, 7, 2, cols)
    assert abs(e.mean()) < 5e-3 and abs(e.var() - 1) < 1e-2
    assert abs((e ** 3).mean()) < 2e-2 and abs((e ** 4).mean() - 3) < 5e-2
    # fraction inside one sigma
    assert abs((np.abs(e) < 1).mean() - 0.682689) < 3e-3
    # neighbouring columns, agents, iterations and seeds are uncorrelated
    others = [noise.normals(3, 7, 3, cols), noise.normals(3, 8, 2, cols), noise.normals(4, 7, 2, cols),
              np.roll(e, 1), np.roll(e, 2)]
    for o in others:
        assert abs(np.corrcoef(e, o)[0, 1]) < 6e-3
    assert np.isfinite(e).all() and np.abs(e).max() < 6.0          # u1 >= 2^-24 bounds the radius


def test_noise_follows_the_normal_law():
    """Kolmogorov-Smirnov distance to the standard normal CDF (scipy's), for one stream and for a column
    taken across many agents and iterations; the integer mix is a bijection of 32-bit words (invertible
    steps: xor-shift, odd multiplier), so distinct counters of one stream give distinct words."""
    from scipy import stats
    e = noise.normals(5, 3, 1, np.arange(200_000))
    assert stats.kstest(e, "norm").statistic < 4e-3                 # 1.36 / sqrt(2e5) = 3.0e-3 at the 5 % level
    across = np.array([noise.normals(5, k, i, np.array([17]))[0] for k in range(60) for i in range(60)])
    assert stats.kstest(across, "norm").statistic < 3.5e-2          # 3600 samples: 2.3e-2 at the 5 % level
    k0, k1 = noise.stream_keys(5, 3, 1)
    words = noise._word(np.arange(1 << 20, dtype=np.uint32), k0, k1)
    assert np.unique(words).size == 1 << 20
    assert np.unique(noise._mix(np.arange(1 << 20, dtype=np.uint32))).size == 1 << 20
    # both halves of the word feed the uniforms: high 24 bits, uniformly spread over 256 buckets
    hist = np.bincount((words >> np.uint32(24)).astype(np.int64), minlength=256)
    assert abs(hist - 4096).max() < 6 * 64                          # binomial sd = 64


def test_noise_is_a_pure_function_of_its_counter():
    cols = np.array([0, 1, 5, 4, 1000001, 1000000, 25_557_031])
    a = noise.normals(11, 49, 30, cols)
    b = np.array([noise.normals(11, 49, 30, np.array([c]))[0] for c in cols])
    assert np.array_equal(a, b)
    # the two members of a pair share a radius: cos^2 + sin^2
    pair = noise.normals(11, 49, 30, np.array([6, 7]))
    k0, k1 = noise.stream_keys(11, 49, 30)
    w1 = noise._word(np.array([6], dtype=np.uint32), k0, k1)[0]
    u1 = (float(w1 >> 8) + 1.0) / 2 ** 24
    assert np.isclose(pair[0] ** 2 + pair[1] ** 2, -2.0 * np.log(u1))


def test_quad_center_noise_free_closed_form():
    """Mean recursion of the averaged-variables lemma with e = z - c: x_bar(k) = c_bar + (1-lr)^k (x_bar(0) - c_bar)."""
    n, d, lr = 6, 9, 0.1
    c = WL.quad_centers(n, d, seed=2)
    x0 = WL.initial_state(n, d, seed=2).astype(np.float64)
    g = losses.make_quad_center_grad(c, 0.0, seed=0)
    for port in (1, 2):
        x, y = x0.copy(), x0.copy()
        for k in range(12):
            x, y = C.dsgd_ceca_step(x, y, k, port, lr, g)
            want = c.mean(0) + (1 - lr) ** (k + 1) * (x0.mean(0) - c.mean(0))
            assert np.allclose(x.mean(0), want, atol=1e-13)


def test_quad_center_fixed_point():
    c = np.tile(WL.quad_centers(1, 5, seed=9), (4, 1))       # all agents share a centre
    g = losses.make_quad_center_grad(c, 0.0, seed=0)
    x = c.astype(np.float64)
    xn, yn = C.dsgd_ceca_step(x, x.copy(), 0, 2, 0.3, g)
    assert np.allclose(xn, c) and np.allclose(yn, c)


def test_quad_center_column_subset_matches_full():
    c = WL.quad_centers(4, 64, seed=3)
    cols = np.array([1, 2, 17, 63])
    full = losses.make_quad_center_grad(c, 0.01, seed=5)
    part = losses.make_quad_center_grad(c[:, cols], 0.01, seed=5, columns=cols)
    z = np.random.default_rng(1).standard_normal((4, 64))
    assert np.array_equal(full(z, 3)[:, cols], part(z[:, cols], 3))


def test_consensus_metrics_closed_form():
    x = np.array([[1.0, 2.0], [3.0, 6.0], [5.0, 4.0]])       # mean (3, 4); deviations (-2,-2), (0,2), (2,0)
    m = consensus.consensus_error(x)
    assert np.allclose(m["mean"], [3.0, 4.0])
    assert np.isclose(m["frob2"], 8 + 4 + 4)
    assert np.isclose(m["residue"], np.sqrt(8) + 2 + 2)
    assert np.isclose(m["max_dev"], np.sqrt(8))
    assert np.isclose(m["mean_norm"], 5.0)


def test_state_consensus_closed_forms():
    """||phi||_F^2 (App. B.3): worked 3-agent example; n * total column variance (library routine);
    and the gossip-only trajectory, where after tau rounds the x part is zero and y_i is the mean of
    the other agents' inputs, so ||phi||^2 = ||u - 1 u_bar^T||_F^2 / (n-1)^2 (matrix-consensus lemma),
    and one round later phi = 0 (Lemma 4.2)."""
    x = np.array([[1.0, 2.0], [3.0, 6.0], [5.0, 4.0]])
    y = np.array([[0.0, 0.0], [2.0, 0.0], [4.0, 3.0]])       # mean (2, 1); deviations (-2,-1), (0,-1), (2,2)
    m = consensus.state_consensus(x, y)
    assert np.isclose(m["x"]["frob2"], 16.0) and np.isclose(m["y"]["frob2"], 5 + 1 + 8)
    assert np.isclose(m["phi2"], 30.0)
    assert np.allclose(m["y"]["mean"], [2.0, 1.0])
    rng = np.random.default_rng(11)
    for n, port in [(5, 2), (6, 1), (31, 2), (100, 1)]:
        u = rng.standard_normal((n, 7)) + 3.0
        w = rng.standard_normal((n, 7))
        m = consensus.state_consensus(u, w)
        assert np.isclose(m["phi2"], n * (np.var(u, axis=0).sum() + np.var(w, axis=0).sum()), rtol=1e-12)
        tau = S.num_rounds(n)
        xs, ys = C.run(u, port, 0.0, None, tau, store32=False)
        m = consensus.state_consensus(xs, ys)
        assert m["x"]["frob2"] < 1e-24
        assert np.isclose(m["phi2"], consensus.consensus_error(u)["frob2"] / (n - 1) ** 2, rtol=1e-10)
        xs, ys = C.gossip_round(xs, ys, 0, port)
        assert consensus.state_consensus(xs, ys)["phi2"] < 1e-24


def test_mirror_mode_reaches_fp32_consensus():
    """The gate used on the device: after tau rounds max_i ||x_i - x_bar|| <= 1e-6 ||x_bar|| with fp32 storage."""
    for n, port in [(5, 2), (6, 1), (31, 2), (100, 1), (100, 2)]:
        x0 = WL.initial_state(n, 512, seed=n)
        x, _ = C.run(x0, port, 0.0, None, S.num_rounds(n), store32=True)
        m = consensus.consensus_error(x)
        assert m["max_dev"] <= 1e-6 * m["mean_norm"]


def test_full_gradient_scale_and_noise_options():
    """grad_scale = 1 with the full batch is the gradient of 1/2 ||A x - b||^2 (the paper's local loss, Sec. 5);
    noise_std adds exactly noise_std * eps(seed, k, agent, column)."""
    n, N, d = 3, 12, 5
    A, b, _ = WL.lsq_data(n, N, d, seed=8)
    idx = WL.full_batch_indices(n, N)
    z = np.random.default_rng(2).standard_normal((n, d))
    g = losses.make_minibatch_grad("lsq", A, b, idx, grad_scale=1.0)(z, 7)
    for i in range(n):
        f = lambda w: 0.5 * float(((A[i].astype(float) @ w - b[i]) ** 2).sum())
        assert np.allclose(g[i], _fd(f, z[i]), rtol=1e-6, atol=1e-6)
    gn = losses.make_minibatch_grad("lsq", A, b, idx, grad_scale=1.0, noise_std=5.0, seed=3)(z, 7)
    for i in range(n):
        assert np.allclose(gn[i] - g[i], 5.0 * noise.normals(3, 7, i, np.arange(d)), atol=1e-12)
    # scale 1/B reproduces the default mean
    gm = losses.make_minibatch_grad("lsq", A, b, idx)(z, 0)
    gs = losses.make_minibatch_grad("lsq", A, b, idx, grad_scale=1.0 / N)(z, 0)
    assert np.allclose(gm, gs, atol=1e-14)


def test_step_size_schedule():
    sp = WL.SPECS["paperlsq258_1p"]
    assert WL.step_size(sp, 0) == 0.02 and WL.step_size(sp, 19) == 0.02
    assert np.isclose(WL.step_size(sp, 20), 0.02 / 1.5) and np.isclose(WL.step_size(sp, 45), 0.02 / 1.5 ** 2)
    assert WL.step_size(WL.SPECS["lsq5_2p"], 150) == 0.01
