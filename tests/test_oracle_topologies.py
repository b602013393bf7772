"""Pins for the comparison-topology oracle (ring, static / one-peer exponential gossip)."""
import numpy as np
import pytest

from oracle import ceca as C
from oracle import consensus
from oracle import schedule as S
from oracle import topologies as T


def _specs(kind, n):
    if kind == "ring":
        return [T.ring(n)]
    if kind == "static":
        return [T.static_exponential(n)]
    return [T.one_peer_exponential(n, k) for k in range(max(T.num_rounds(n), 1))]


@pytest.mark.parametrize("kind", ["ring", "static", "onepeer"])
@pytest.mark.parametrize("n", [1, 2, 3, 5, 6, 8, 31, 100, 130])
def test_doubly_stochastic_and_three_forms_agree(kind, n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((n, 3))
    for m in _specs(kind, n):
        W = T.mix_matrix(n, m)
        assert np.allclose(W.sum(axis=1), 1.0) and np.allclose(W.sum(axis=0), 1.0) and (W >= 0).all()
        per_agent = T.mix_round(x, m)
        assert np.allclose(per_agent, W @ x, atol=1e-14)
        # circular convolution (textbook): x+ = c * x with c[s] the weight of the agent s places back
        c = np.zeros(n)
        c[0] += m.w_self
        for s, w in zip(m.shifts, m.weights):
            c[s % n] += w
        conv = np.fft.ifft(np.fft.fft(c)[:, None] * np.fft.fft(x, axis=0), axis=0).real
        assert np.allclose(per_agent, conv, atol=1e-12)
        assert np.allclose(per_agent.mean(axis=0), x.mean(axis=0), atol=1e-14)    # column-stochastic


def test_direction_and_weights_on_a_one_hot_input():
    n = 7
    x = np.zeros((n, 1)); x[2, 0] = 1.0
    assert np.allclose(T.mix_round(x, T.one_peer_exponential(n, 1))[:, 0], [0, 0, .5, 0, .5, 0, 0])   # 2 -> 2 + 2
    assert np.allclose(T.mix_round(x, T.ring(n))[:, 0], [0, 1 / 3, 1 / 3, 1 / 3, 0, 0, 0])
    got = T.mix_round(x, T.static_exponential(n))[:, 0]             # tau = 3: to 2, 3, 4, 6
    assert np.allclose(got, [0, 0, .25, .25, .25, 0, .25])


@pytest.mark.parametrize("n", [2, 4, 8, 16, 64, 256])
def test_one_peer_exponential_is_exact_and_is_ceca_for_powers_of_two(n):
    """Sec. 1: for n a power of two, log2 n one-peer exponential rounds average exactly; there CECA's
    two-port rounds are the same rounds (derived from Eqs. (2), (3), (5))."""
    rng = np.random.default_rng(n)
    u = rng.standard_normal((n, 4))
    tau = T.num_rounds(n)
    x = u.copy()
    cx, cy = u.copy(), u.copy()
    for k in range(tau):
        x = T.mix_round(x, T.one_peer_exponential(n, k))
        cx, cy = C.gossip_round(cx, cy, k, 2, store32=False)
        assert np.allclose(x, cx, atol=1e-14)
    assert np.allclose(x, u.mean(axis=0), atol=1e-13)


def test_ring_eigenvalues_are_the_cosines():
    n = 12
    ev = np.sort(np.linalg.eigvalsh(T.mix_matrix(n, T.ring(n))))
    want = np.sort(1 / 3 + 2 / 3 * np.cos(2 * np.pi * np.arange(n) / n))
    assert np.allclose(ev, want, atol=1e-12)


@pytest.mark.parametrize("n", [130, 1026])
def test_only_ceca_reaches_consensus_in_finitely_many_rounds(n):
    """Sec. 5, consensus comparison: at n = 130 and n = 1026 CECA is at the exact mean after tau rounds;
    ring, static and one-peer exponential gossip still are not after 3 tau."""
    u = np.random.default_rng(n).standard_normal((n, 2))
    tau = S.num_rounds(n)
    x, _ = C.run(u, 1, 0.0, None, tau, store32=False)
    assert consensus.consensus_error(x)["residue"] < 1e-10 * n
    start = consensus.consensus_error(u)["residue"]
    for kind in ("ring", "static", "onepeer"):
        res = consensus.consensus_error(T.run(u, _specs(kind, n), 3 * tau, store32=False))["residue"]
        assert 1e-9 * start < res < start, kind
