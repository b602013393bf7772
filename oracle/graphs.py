"""Gossip averaging over arbitrary graphs -- TEST INFRASTRUCTURE ONLY.

Table 1 of the paper lists, beside the circulant topologies of oracle/topologies.py, graphs whose mixing
step is not shift-invariant: grid, torus, hypercube (and any graph a user brings).  The paper defines none
of them; the definitions below are the textbook ones of decentralized averaging, restated:

    x_i+ = W_ii x_i + sum_{j in N(i)} W_ij x_j,                 W symmetric, doubly stochastic,

  Metropolis weights of an undirected graph:  W_ij = 1 / (1 + max(deg i, deg j)) for every edge,
                                               W_ii = 1 - sum_j W_ij
  hypercube (n = 2^tau) ....... i ~ i xor 2^b for every bit b; every vertex has degree tau, so the
                                Metropolis weights are all 1/(tau + 1)
  one-peer hypercube, round k . the single edge i ~ i xor 2^(k mod tau), weights 1/2, 1/2: exact
                                averaging after tau rounds (pairwise averaging along every bit)
  2-D torus r x c ............. (a, b) ~ (a +- 1 mod r, b), (a, b +- 1 mod c); vertex a*c + b
  2-D grid r x c .............. the same without wrap-around

A round is stored as a neighbour table: nbr[i, j] (0-based vertex), w[i, j], w_self[i], j < m, rows with
fewer than m neighbours padded with (i, 0.0).

Pin status: symmetry and double stochasticity; the dense product W x against the row-by-row form; closed-form
spectra (hypercube: 1 - 2k/(tau+1) with multiplicity C(tau, k); torus with equal degrees: sums of cosines);
exact averaging of the one-peer hypercube in tau rounds; equality with the circulant oracle on a ring.  The
paper prints no values for these graphs: *parity unpinned by the paper* beyond that.
"""
from __future__ import annotations

from typing import Iterable, List, Sequence, Tuple

import numpy as np

Table = Tuple[np.ndarray, np.ndarray, np.ndarray]      # nbr (n, m) int, w (n, m) float64, w_self (n,) float64


def _table(n: int, rows: Sequence[Sequence[Tuple[int, float]]]) -> Table:
    m = max(1, max(len(r) for r in rows))
    nbr = np.empty((n, m), dtype=np.int64)
    w = np.zeros((n, m), dtype=np.float64)
    for i, r in enumerate(rows):
        nbr[i, :] = i
        for j, (v, wt) in enumerate(r):
            nbr[i, j] = v
            w[i, j] = wt
    return nbr, w, 1.0 - w.sum(axis=1)


def metropolis(n: int, edges: Iterable[Tuple[int, int]]) -> Table:
    """Metropolis weights of the undirected simple graph with the given edges."""
    adj: List[set] = [set() for _ in range(n)]
    for a, b in edges:
        if a != b:
            adj[a].add(b)
            adj[b].add(a)
    rows = [[(j, 1.0 / (1.0 + max(len(adj[i]), len(adj[j])))) for j in sorted(adj[i])] for i in range(n)]
    return _table(n, rows)


def hypercube_edges(tau: int):
    return [(i, i ^ (1 << b)) for i in range(1 << tau) for b in range(tau) if i < i ^ (1 << b)]


def hypercube(tau: int) -> Table:
    return metropolis(1 << tau, hypercube_edges(tau))


def one_peer_hypercube(tau: int, k: int) -> Table:
    n = 1 << tau
    if tau == 0:
        return _table(1, [[]])
    b = k % tau
    return _table(n, [[(i ^ (1 << b), 0.5)] for i in range(n)])


def torus_edges(r: int, c: int):
    e = []
    for a in range(r):
        for b in range(c):
            e.append((a * c + b, ((a + 1) % r) * c + b))
            e.append((a * c + b, a * c + (b + 1) % c))
    return e


def grid_edges(r: int, c: int):
    e = []
    for a in range(r):
        for b in range(c):
            if a + 1 < r:
                e.append((a * c + b, (a + 1) * c + b))
            if b + 1 < c:
                e.append((a * c + b, a * c + b + 1))
    return e


def graph_round(x: np.ndarray, t: Table) -> np.ndarray:
    """The definition, vertex by vertex, in fp64."""
    nbr, w, w_self = t
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    for i in range(x.shape[0]):
        acc = w_self[i] * x[i]
        for j in range(nbr.shape[1]):
            acc = acc + w[i, j] * x[nbr[i, j]]
        out[i] = acc
    return out


def dense(t: Table) -> np.ndarray:
    nbr, w, w_self = t
    n = nbr.shape[0]
    W = np.zeros((n, n))
    for i in range(n):
        W[i, i] += w_self[i]
        for j in range(nbr.shape[1]):
            W[i, nbr[i, j]] += w[i, j]
    return W


def run(x0: np.ndarray, tables: Sequence[Table], rounds: int, k0: int = 0, store32: bool = True) -> np.ndarray:
    """rounds rounds, round t using tables[(k0 + t) mod len(tables)]; store32 rounds the state to fp32 after
    every round (the precision the device stores)."""
    x = np.asarray(x0, dtype=np.float64)
    for t in range(rounds):
        x = graph_round(x, tables[(k0 + t) % len(tables)])
        if store32:
            x = x.astype(np.float32).astype(np.float64)
    return x
