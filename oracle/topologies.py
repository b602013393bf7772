"""Shift-invariant gossip averaging over the comparison topologies -- TEST INFRASTRUCTURE ONLY.

The paper compares CECA's finite-time consensus with ring, static exponential and one-peer
exponential gossip (Table 1; Sec. 5, consensus comparison at n = 130 and n = 1026) but defines none
of them: the definitions are those of the works it cites for them, restated here.  Every one is a
circulant mixing step on x alone,

    x_i+ = w_self x_i + sum_j w_j x_{(i - s_j) mod n},          rows 0-based,

  ring ................ s = (1, n-1), all three weights 1/3 (n = 2: 1/2, 1/2; n = 1: identity)
  static exponential .. s = (2^0, 2^1, ..., 2^(tau-1)), every weight 1/(tau+1), tau = ceil(log2 n)
  one-peer exponential  round k: s = (2^(k mod tau)), weights 1/2, 1/2

The direction "receive from i - s" is the one CECA's two-port rounds use (App. B.1.1), so that the
one-peer exponential rounds are exactly CECA's rounds when n is a power of two.

Pin status: row and column sums; agreement of the per-agent form, the dense matrix and the FFT
(circular-convolution) form; exact averaging by one-peer exponential in log2 n rounds when n is a power
of two (Sec. 1) and its equality with CECA there; the ring's cosine eigenvalues.  The paper prints no
values for these topologies: *parity unpinned by the paper* beyond that.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Mix:
    shifts: Tuple[int, ...]
    weights: Tuple[float, ...]      # weight of x_{i - shifts[j]}
    w_self: float


def num_rounds(n: int) -> int:
    return (n - 1).bit_length()


def ring(n: int) -> Mix:
    if n == 1:
        return Mix((), (), 1.0)
    if n == 2:
        return Mix((1,), (0.5,), 0.5)
    return Mix((1, n - 1), (1.0 / 3.0, 1.0 / 3.0), 1.0 / 3.0)


def static_exponential(n: int) -> Mix:
    tau = num_rounds(n)
    w = 1.0 / (tau + 1)
    return Mix(tuple(1 << j for j in range(tau)), (w,) * tau, w)


def one_peer_exponential(n: int, k: int) -> Mix:
    tau = num_rounds(n)
    if tau == 0:
        return Mix((), (), 1.0)
    return Mix((1 << (k % tau),), (0.5,), 0.5)


def mix_round(x: np.ndarray, m: Mix) -> np.ndarray:
    """The definition, agent by agent, in fp64."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    out = np.empty_like(x)
    for i in range(n):
        acc = m.w_self * x[i]
        for s, w in zip(m.shifts, m.weights):
            acc = acc + w * x[(i - s) % n]
        out[i] = acc
    return out


def mix_matrix(n: int, m: Mix) -> np.ndarray:
    """Dense W with x+ = W x, built entry by entry."""
    W = np.zeros((n, n))
    for i in range(n):
        W[i, i] += m.w_self
        for s, w in zip(m.shifts, m.weights):
            W[i, (i - s) % n] += w
    return W


def run(x0: np.ndarray, specs: Sequence[Mix], rounds: int, k0: int = 0, store32: bool = True) -> np.ndarray:
    """rounds rounds, round t using specs[(k0 + t) mod len(specs)]; store32 rounds the state to fp32
    after every round (the precision the device stores)."""
    x = np.asarray(x0, dtype=np.float64)
    for t in range(rounds):
        x = mix_round(x, specs[(k0 + t) % len(specs)])
        if store32:
            x = x.astype(np.float32).astype(np.float64)
    return x
