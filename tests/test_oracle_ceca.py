"""Pins for oracle/ceca.py: the paper's printed n = 6 example, window invariants, the exact
tau-round matrix product for every n <= 64, Lemma 4.1, the mean lemma (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ceca as C
from oracle import schedule as S


def _read_value_table(lines):
    out = {}
    for ln in lines:
        f = ln.split()
        vals = [float(v) for v in f[1:]]
        out[int(f[0])] = (np.array(vals[0::2]), np.array(vals[1::2]))
    return out


@pytest.mark.parametrize("port,name", [(2, "ceca_n6_values_2p.txt"), (1, "ceca_n6_values_1p.txt")])
def test_n6_value_tables(golden, port, name):
    tab = _read_value_table(golden(name))
    x, y = tab[0][0][:, None].copy(), tab[0][1][:, None].copy()
    for r in range(3):
        x, y = C.gossip_round(x, y, r, port)
        assert np.allclose(x[:, 0], tab[r + 1][0], atol=1e-12), (port, r)
        assert np.allclose(y[:, 0], tab[r + 1][1], atol=1e-12), (port, r)
        xd, yd = C.gossip_round_dense(tab[r][0][:, None], tab[r][1][:, None], r, port)
        assert np.allclose(xd[:, 0], tab[r + 1][0], atol=1e-12)
        assert np.allclose(yd[:, 0], tab[r + 1][1], atol=1e-12)


def _read_coeff(lines):
    out, i = {}, 0
    while i < len(lines):
        name, rnd = lines[i].split()
        rows = [[Fraction(v) for v in lines[i + 1 + p].split()] for p in range(6)]
        out[(name, int(rnd))] = rows
        i += 7
    return out


def _exact_product(n, port, rounds):
    """W^(rounds-1) ... W^(0) in exact rationals (product order of App. A), rounds taken cyclically."""
    tau = S.num_rounds(n)
    M = np.array([[Fraction(int(p == q)) for q in range(2 * n)] for p in range(2 * n)], dtype=object)
    for k in range(rounds):
        W, _ = C.mixing_matrices(n, k % tau, port)
        # sparse left-multiplication keeps exact arithmetic cheap: each row of W has <= 2 entries
        new = np.empty_like(M)
        for p in range(2 * n):
            nz = [(q, W[p, q]) for q in range(2 * n) if W[p, q] != 0]
            new[p] = sum((w * M[q] for q, w in nz[1:]), nz[0][1] * M[nz[0][0]])
        M = new
    return M


@pytest.mark.parametrize("port,name", [(2, "ceca_n6_coeff_2p.txt"), (1, "ceca_n6_coeff_1p.txt")])
def test_n6_coefficient_matrices(golden, port, name):
    coeff = _read_coeff(golden(name))
    for s in (1, 2, 3):
        M = _exact_product(6, port, s)
        # the product maps [u; J0] to [I^(s); J^(s)]; with J^(0) = 0 only its left blocks matter
        assert [[M[p, q] for q in range(6)] for p in range(6)] == coeff[("I", s)]
        assert [[M[6 + p, q] for q in range(6)] for p in range(6)] == coeff[("J", s)]


def _scaled_int_product(n, port, rounds):
    """Brute-force dense product with every W^(r) scaled to an integer matrix (exact in int64 for n <= 64)."""
    tau = S.num_rounds(n)
    M = np.eye(2 * n, dtype=np.int64)
    scale = 1
    for k in range(rounds):
        r = k % tau
        W, _ = C.mixing_matrices(n, r, port)
        D = 2 * (2 * S.window_sizes(n)[r] + 1)
        Wi = np.array([[int(v * D) for v in row] for row in W], dtype=np.int64)
        assert all((v * D).denominator == 1 for row in W for v in row)
        M = Wi @ M
        scale *= D
    return M, scale


@pytest.mark.parametrize("n", range(2, 65))
def test_tau_round_product_two_port(n):
    _check_product(n, 2)


@pytest.mark.parametrize("n", range(2, 65, 2))
def test_tau_round_product_one_port(n):
    _check_product(n, 1)


def _check_product(n, port):
    tau = S.num_rounds(n)
    ones = np.ones((n, n), dtype=np.int64)
    eye = np.eye(n, dtype=np.int64)
    M, sc = _scaled_int_product(n, port, tau)
    assert sc < 2 ** 52
    # matrix-consensus lemma, first identity: [[11^T/n, 0], [(11^T - I)/(n-1), 0]]
    assert np.array_equal(M[:n, :n] * n, sc * ones)
    assert np.array_equal(M[n:, :n] * (n - 1), sc * (ones - eye))
    assert not M[:, n:].any()
    # one more round: both left blocks are 11^T / n (second identity, Lemma 4.2)
    M, sc = _scaled_int_product(n, port, tau + 1)
    assert np.array_equal(M[:n, :n] * n, sc * ones)
    assert np.array_equal(M[n:, :n] * n, sc * ones)
    assert not M[:, n:].any()


@pytest.mark.parametrize("n", [2, 3, 5, 6, 7, 12, 31, 33, 64])
def test_window_invariant_two_port(n):
    """Eq. (4) / proof of the matrix-consensus lemma: after s+1 rounds the x block is the banded
    circulant 1/(n_{s+1}+1) on i-j in {0..n_{s+1}}, the y block 1/n_{s+1} on {1..n_{s+1}}."""
    nr = S.window_sizes(n)
    for s in range(S.num_rounds(n)):
        M = _exact_product(n, 2, s + 1)
        m = nr[s + 1]
        for i in range(n):
            for j in range(n):
                dlt = (i - j) % n
                assert M[i, j] == (Fraction(1, m + 1) if dlt <= m else 0)
                assert M[n + i, j] == (Fraction(1, m) if 1 <= dlt <= m else 0)


@pytest.mark.parametrize("n", [2, 6, 10, 12, 30, 34, 64])
def test_window_invariant_one_port(n):
    """App. B.1.2: odd agents (1-based) hold the window ahead of them, even agents the window behind."""
    nr = S.window_sizes(n)
    for s in range(S.num_rounds(n)):
        M = _exact_product(n, 1, s + 1)
        m = nr[s + 1]
        for i in range(n):
            sign = 1 if (i + 1) % 2 == 1 else -1
            for j in range(n):
                dlt = (sign * (j - i)) % n
                assert M[i, j] == (Fraction(1, m + 1) if dlt <= m else 0)
                assert M[n + i, j] == (Fraction(1, m) if 1 <= dlt <= m else 0)


@pytest.mark.parametrize("n,port", [(5, 2), (6, 1), (6, 2), (31, 2), (30, 1), (100, 2), (100, 1)])
def test_lemma_4_1_properties(n, port):
    blockmean = np.kron(np.eye(2), np.ones((n, n)) / n)
    for r in range(S.num_rounds(n)):
        for M in C.mixing_matrices(n, r, port):
            assert all(sum(row) == 1 for row in M)                    # row stochastic
            Mf = C.to_float(M)
            assert np.linalg.norm(Mf, 2) <= np.sqrt(2) + 1e-12         # ||W|| <= sqrt 2
            assert np.allclose(Mf @ blockmean, blockmean @ Mf, atol=1e-14)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_power_of_two_is_one_peer_exponential(n):
    """Derived, not stated by the paper: for n = 2^tau every delta_r is 1, so x+ = (x_i + x_{i-2^r})/2."""
    rng = np.random.default_rng(n)
    x = rng.standard_normal((n, 3))
    y = rng.standard_normal((n, 3))
    for r in range(S.num_rounds(n)):
        xn, _ = C.gossip_round(x, y, r, 2)
        assert np.allclose(xn, 0.5 * (x + np.roll(x, 1 << r, axis=0)), atol=1e-15)


@pytest.mark.parametrize("n,port", [(3, 2), (5, 2), (6, 1), (6, 2), (31, 2), (30, 1), (100, 1), (100, 2), (258, 1)])
def test_exact_consensus_and_y_limit(n, port):
    rng = np.random.default_rng(7 * n + port)
    u = rng.standard_normal((n, 4))
    x, y = u.copy(), rng.standard_normal((n, 4))      # any y(0): round 0 overwrites it (b = 0)
    tau = S.num_rounds(n)
    mean = u.mean(axis=0)
    for r in range(tau):
        x, y = C.gossip_round(x, y, r, port)
        assert np.allclose(x.mean(axis=0), mean, atol=1e-13)           # mean of x never moves
        assert np.allclose(y.mean(axis=0), mean, atol=1e-13)           # and y joins it after round 0
    assert np.allclose(x, mean, atol=1e-13)
    assert np.allclose(y, (n * mean - u) / (n - 1), atol=1e-13)       # J^(tau): mean of the others
    x, y = C.gossip_round(x, y, 0, port)
    assert np.allclose(x, mean, atol=1e-13) and np.allclose(y, mean, atol=1e-13)


def _toy_grad(seed):
    def grad(z, k):
        rng = np.random.default_rng([seed, k])
        Q = rng.standard_normal((z.shape[0], z.shape[1]))
        return np.tanh(z) * (1.0 + 0.1 * Q) + 0.3 * Q      # any per-agent map will do
    return grad


@pytest.mark.parametrize("n,port", [(2, 2), (5, 2), (6, 1), (6, 2), (13, 2), (14, 1)])
def test_two_codings_agree_and_mean_lemma(n, port):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((n, 5))
    y = x.copy()
    lr = 0.07
    grad = _toy_grad(n)
    xd, yd = x.copy(), y.copy()
    for k in range(3 * S.num_rounds(n) + 1):
        r = k % S.num_rounds(n)
        z = x if S.exchanged(n, r) == "x" else y
        ebar = grad(z, k).mean(axis=0)
        xbar = x.mean(axis=0)
        assert np.allclose(x.mean(axis=0), y.mean(axis=0), atol=1e-13)      # x_bar = y_bar
        x, y = C.dsgd_ceca_step(x, y, k, port, lr, grad)
        xd, yd = C.dsgd_ceca_step_dense(xd, yd, k, port, lr, grad)
        assert np.allclose(x, xd, atol=1e-13) and np.allclose(y, yd, atol=1e-13)
        assert np.allclose(x.mean(axis=0), xbar - lr * ebar, atol=1e-13)    # x_bar+ = x_bar - lr e_bar


def test_zero_gradient_step_is_gossip_round():
    rng = np.random.default_rng(0)
    x, y = rng.standard_normal((6, 3)), rng.standard_normal((6, 3))
    zero = lambda z, k: np.zeros_like(z)
    for k in range(3):
        for port in (1, 2):
            a = C.dsgd_ceca_step(x, y, k, port, 0.5, zero)
            b = C.gossip_round(x, y, k, port)
            assert np.allclose(a[0], b[0], atol=1e-15) and np.allclose(a[1], b[1], atol=1e-15)


def test_planted_mistakes_are_caught(monkeypatch, golden):
    """The pins must fail on plausible slips: a reversed shift, swapped weights, the wrong variable sent."""
    tab = _read_value_table(golden("ceca_n6_values_2p.txt"))

    def run():
        x, y = tab[0][0][:, None].copy(), tab[0][1][:, None].copy()
        for r in range(3):
            x, y = C.gossip_round(x, y, r, 2)
            if not (np.allclose(x[:, 0], tab[r + 1][0]) and np.allclose(y[:, 0], tab[r + 1][1])):
                return False
        return True

    assert run()
    good_peers = S.peers
    monkeypatch.setattr(S, "peers", lambda n, r, port: [(2 * i - p) % n for i, p in enumerate(good_peers(n, r, port))])
    assert not run()                                   # receive from i+s instead of i-s
    monkeypatch.setattr(S, "peers", good_peers)
    good_bits = S.delta_bits
    monkeypatch.setattr(S, "delta_bits", lambda n: good_bits(n)[::-1] if n != 6 else [1, 1, 0])
    assert not run()                                   # bits read in the wrong order
    monkeypatch.setattr(S, "delta_bits", good_bits)
    assert run()
