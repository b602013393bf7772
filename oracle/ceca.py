"""CECA gossip round and the DSGD-CECA step, fp64 -- TEST INFRASTRUCTURE ONLY.

Two independent codings of the same update:

  * per agent, straight from the recursions of Sec. 3.1 / 3.2 (gossip) and from
    Algorithm 1 with Eqs. (8), (9) (DSGD-CECA, Sec. 4.1);
  * dense: the 2n x 2n mixing matrices W, W_g of Eqs. (10), (11) applied as in
    Eq. (12), with the communication matrix P built entry by entry from the
    congruences of Eqs. (5)-(7).

State: x, y are (n, d) float64 arrays, row = agent (App. A).  "Mirror mode"
(`store32=True`) rounds the new state to float32 once per step, which is the
precision the device keeps it in; all arithmetic inside a step stays fp64.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Callable, Optional, Tuple

import numpy as np

from . import schedule as S


def _store(a: np.ndarray, store32: bool) -> np.ndarray:
    return a.astype(np.float32).astype(np.float64) if store32 else a


# ---------------------------------------------------------------------------
# per-agent coding
# ---------------------------------------------------------------------------

def gossip_round(x: np.ndarray, y: np.ndarray, r: int, port: int, store32: bool = False
                 ) -> Tuple[np.ndarray, np.ndarray]:
    """One CECA round on (I, J) = (x, y) (Sec. 3.1 "Main recursions"; Sec. 3.2 for one port)."""
    n = x.shape[0]
    if n == 1:
        return x.copy(), y.copy()
    dlt = S.delta_bits(n)[r]
    m = S.window_sizes(n)[r]
    src = S.peers(n, r, port)
    xn = np.empty_like(x)
    yn = np.empty_like(y)
    for i in range(n):
        w = src[i]
        if dlt == 1:
            xn[i] = 0.5 * x[i] + 0.5 * x[w]
            yn[i] = (m / (2 * m + 1)) * y[i] + ((m + 1) / (2 * m + 1)) * x[w]
        else:
            xn[i] = ((m + 1) / (2 * m + 1)) * x[i] + (m / (2 * m + 1)) * y[w]
            yn[i] = 0.5 * y[i] + 0.5 * y[w]
    return _store(xn, store32), _store(yn, store32)


GradFn = Callable[[np.ndarray, int], np.ndarray]  # (z (n,d), k) -> e (n,d): one stochastic gradient per agent


def dsgd_ceca_step(x: np.ndarray, y: np.ndarray, k: int, port: int, lr: float, grad: GradFn,
                   store32: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Iteration k of Algorithm 1: r = k mod tau, gradient at z (x if delta_r = 1 else y),
    every agent sends z_i - lr*e_i, then Eqs. (8), (9)."""
    n = x.shape[0]
    tau = S.num_rounds(n)
    if tau == 0:
        # a single agent has nobody to talk to: plain SGD, y follows x
        e = grad(x, k)
        xn = x - lr * e
        return _store(xn, store32), _store(xn.copy(), store32)
    r = k % tau
    a, b = (float(w) for w in S.weights(n, r))
    z = x if S.exchanged(n, r) == "x" else y
    src = S.peers(n, r, port)
    e = grad(z, k)
    v = z - lr * e                       # what each agent sends
    xn = np.empty_like(x)
    yn = np.empty_like(y)
    for i in range(n):
        xn[i] = a * (x[i] - lr * e[i]) + (1.0 - a) * v[src[i]]      # Eq. (8)
        yn[i] = b * (y[i] - lr * e[i]) + (1.0 - b) * v[src[i]]      # Eq. (9)
    return _store(xn, store32), _store(yn, store32)


# ---------------------------------------------------------------------------
# dense coding
# ---------------------------------------------------------------------------

def comm_matrix(n: int, r: int, port: int) -> np.ndarray:
    """P = Q^(r) as an n x n 0/1 integer matrix, Q_{i,j} = 1 iff j sends to i, decided
    entry by entry from the conditions of Eqs. (5), (6) (two ports) and Eq. (7) (one port)."""
    dlt = S.delta_bits(n)[r]
    m = S.window_sizes(n)[r]
    Q = np.zeros((n, n), dtype=np.int64)
    for i in range(1, n + 1):
        for j in range(1, n + 1):
            if port == 2:
                hit = (i - j - (m + dlt)) % n == 0
            elif port == 1:
                if n % 2:
                    raise ValueError("CECA-1P is defined for even n only")
                off = 2 * m + 1
                hit = ((j - i - off) % n == 0) if i % 2 == 1 else ((j - i + off) % n == 0)
            else:
                raise ValueError("port must be 1 or 2")
            if hit:
                Q[i - 1, j - 1] = 1
    return Q


def mixing_matrices(n: int, r: int, port: int):
    """(W, W_g) of Eqs. (10), (11) as 2n x 2n object arrays of exact Fractions."""
    dlt = S.delta_bits(n)[r]
    m = S.window_sizes(n)[r]
    P = comm_matrix(n, r, port)
    I = np.eye(n, dtype=np.int64)
    half = Fraction(1, 2)
    lo = Fraction(m, 2 * m + 1)
    hi = Fraction(m + 1, 2 * m + 1)

    def blk(cI, cP):
        # cI * I_n + cP * P, entries kept as exact Fractions
        M = np.full((n, n), Fraction(0), dtype=object)
        for p, q in zip(*np.nonzero(I)):
            M[p, q] += cI
        for p, q in zip(*np.nonzero(P)):
            M[p, q] += cP
        return M

    zero = blk(Fraction(0), Fraction(0))
    if dlt == 1:
        W = np.block([[blk(half, half), zero], [blk(Fraction(0), hi), blk(lo, Fraction(0))]])
        Wg = np.block([[blk(half, half), zero], [blk(lo, hi), zero]])
    else:
        W = np.block([[blk(hi, Fraction(0)), blk(Fraction(0), lo)], [zero, blk(half, half)]])
        Wg = np.block([[zero, blk(hi, lo)], [zero, blk(half, half)]])
    return W, Wg


def to_float(M) -> np.ndarray:
    return np.array([[float(v) for v in row] for row in M], dtype=np.float64)


def dsgd_ceca_step_dense(x: np.ndarray, y: np.ndarray, k: int, port: int, lr: float, grad: GradFn,
                         store32: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (12): [x; y]+ = W [x; y] - lr * W_g [g; h] with g, h the gradients at x and at y."""
    n = x.shape[0]
    tau = S.num_rounds(n)
    r = k % tau
    W, Wg = mixing_matrices(n, r, port)
    Wf, Wgf = to_float(W), to_float(Wg)
    g = grad(x, k)
    h = grad(y, k)
    new = Wf @ np.vstack([x, y]) - lr * (Wgf @ np.vstack([g, h]))
    return _store(new[:n], store32), _store(new[n:], store32)


def gossip_round_dense(x: np.ndarray, y: np.ndarray, r: int, port: int) -> Tuple[np.ndarray, np.ndarray]:
    n = x.shape[0]
    W, _ = mixing_matrices(n, r, port)
    new = to_float(W) @ np.vstack([x, y])
    return new[:n], new[n:]


def run(x0: np.ndarray, port: int, lr: float, grad: Optional[GradFn], iters: int, store32: bool = True,
        y0: Optional[np.ndarray] = None, k0: int = 0):
    """`iters` iterations of Algorithm 1 from x(0) = x0, y(0) = x0 (its initialisation line);
    grad = None runs gradient-free gossip rounds instead."""
    x = _store(np.asarray(x0, dtype=np.float64), store32)
    y = x.copy() if y0 is None else _store(np.asarray(y0, dtype=np.float64), store32)
    n = x.shape[0]
    tau = S.num_rounds(n)
    for k in range(k0, k0 + iters):
        if grad is None:
            if tau:
                x, y = gossip_round(x, y, k % tau, port, store32)
        else:
            x, y = dsgd_ceca_step(x, y, k, port, lr, grad, store32)
    return x, y
