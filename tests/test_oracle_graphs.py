"""Pins for the general-graph gossip oracle (Metropolis weights; hypercube, torus, grid of Table 1)."""
from math import comb

import numpy as np
import pytest

from oracle import graphs as G
from oracle import topologies as T


def _cases():
    return {"hypercube4": G.hypercube(4), "torus3x5": G.metropolis(15, G.torus_edges(3, 5)),
            "grid4x3": G.metropolis(12, G.grid_edges(4, 3)), "path5": G.metropolis(5, [(0, 1), (1, 2), (2, 3), (3, 4)]),
            "star6": G.metropolis(6, [(0, j) for j in range(1, 6)]), "one_peer_cube": G.one_peer_hypercube(3, 1)}


@pytest.mark.parametrize("name", sorted(_cases()))
def test_symmetric_doubly_stochastic_and_forms_agree(name):
    t = _cases()[name]
    W = G.dense(t)
    assert np.allclose(W, W.T) and (W >= -1e-15).all()
    assert np.allclose(W.sum(axis=1), 1.0) and np.allclose(W.sum(axis=0), 1.0)
    x = np.random.default_rng(1).standard_normal((W.shape[0], 4))
    got = G.graph_round(x, t)
    assert np.allclose(got, W @ x, atol=1e-14)
    assert np.allclose(got.mean(axis=0), x.mean(axis=0), atol=1e-14)


def test_metropolis_weights_on_hand_made_graphs():
    # path 0-1-2: degrees 1, 2, 1: both edges weigh 1/3; the ends keep 2/3, the middle 1/3
    W = G.dense(G.metropolis(3, [(0, 1), (1, 2)]))
    assert np.allclose(W, [[2 / 3, 1 / 3, 0], [1 / 3, 1 / 3, 1 / 3], [0, 1 / 3, 2 / 3]])
    # star with 5 leaves: every edge 1/6, the hub keeps 1/6, a leaf 5/6
    W = G.dense(G.metropolis(6, [(0, j) for j in range(1, 6)]))
    assert np.isclose(W[0, 0], 1 / 6) and np.allclose(W[0, 1:], 1 / 6) and np.allclose(np.diag(W)[1:], 5 / 6)
    # 3 x 3 grid: corner degree 2, side 3, centre 4
    W = G.dense(G.metropolis(9, G.grid_edges(3, 3)))
    assert np.isclose(W[0, 1], 1 / 4) and np.isclose(W[1, 4], 1 / 5) and np.isclose(W[0, 0], 1 / 2) and np.isclose(W[4, 4], 1 / 5)
    # duplicate and reversed edges, self loops: ignored
    assert np.allclose(G.dense(G.metropolis(3, [(0, 1), (1, 0), (1, 1), (1, 2), (1, 2)])), G.dense(G.metropolis(3, [(0, 1), (1, 2)])))


@pytest.mark.parametrize("tau", [1, 2, 3, 5])
def test_hypercube_spectrum_closed_form(tau):
    ev = np.sort(np.linalg.eigvalsh(G.dense(G.hypercube(tau))))
    want = np.sort(np.concatenate([[1.0 - 2.0 * k / (tau + 1)] * comb(tau, k) for k in range(tau + 1)]))
    assert np.allclose(ev, want, atol=1e-12)


@pytest.mark.parametrize("r,c", [(3, 3), (4, 5), (3, 7)])
def test_torus_spectrum_closed_form(r, c):
    """Every vertex of an r x c torus (r, c >= 3) has degree 4: W = (I + shifts) / 5, eigenvalues (1 + 2 cos + 2 cos) / 5."""
    ev = np.sort(np.linalg.eigvalsh(G.dense(G.metropolis(r * c, G.torus_edges(r, c)))))
    want = np.sort([(1 + 2 * np.cos(2 * np.pi * a / r) + 2 * np.cos(2 * np.pi * b / c)) / 5 for a in range(r) for b in range(c)])
    assert np.allclose(ev, want, atol=1e-12)


@pytest.mark.parametrize("tau", [0, 1, 2, 4, 6])
def test_one_peer_hypercube_averages_exactly_in_tau_rounds(tau):
    n = 1 << tau
    x0 = np.random.default_rng(tau).standard_normal((n, 3))
    tabs = [G.one_peer_hypercube(tau, k) for k in range(max(tau, 1))]
    x = G.run(x0, tabs, tau, store32=False)
    assert np.allclose(x, x0.mean(axis=0), atol=1e-14)
    if tau >= 2:
        assert not np.allclose(G.run(x0, tabs, tau - 1, store32=False), x0.mean(axis=0), atol=1e-6)
    P = np.eye(n)
    for k in range(tau):
        P = G.dense(tabs[k]) @ P
    assert np.allclose(P, np.full((n, n), 1.0 / n), atol=1e-15)


@pytest.mark.parametrize("n", [3, 8, 31])
def test_ring_as_a_graph_equals_the_circulant_oracle(n):
    t = G.metropolis(n, [(i, (i + 1) % n) for i in range(n)])
    assert np.allclose(G.dense(t), T.mix_matrix(n, T.ring(n)), atol=1e-15)
    x0 = np.random.default_rng(n).standard_normal((n, 5))
    assert np.allclose(G.run(x0, [t], 7, store32=False), T.run(x0, [T.ring(n)], 7, store32=False), atol=1e-13)


def test_padding_and_direction():
    # a directed table (not symmetric): vertex 0 takes everything from vertex 2, the others keep their value
    nbr = np.array([[2], [1], [2]]); w = np.array([[1.0], [0.0], [0.0]]); ws = np.array([0.0, 1.0, 1.0])
    x = np.array([[1.0], [10.0], [100.0]])
    assert np.array_equal(G.graph_round(x, (nbr, w, ws)), [[100.0], [10.0], [100.0]])
    # a vertex with fewer neighbours than the table is wide is padded with itself at weight zero
    nbr, w, ws = G.metropolis(3, [(0, 1), (1, 2)])
    assert nbr.shape == (3, 2) and nbr[0, 1] == 0 and w[0, 1] == 0.0 and nbr[2, 1] == 2 and w[2, 1] == 0.0
