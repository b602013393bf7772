"""CECA round schedule, integer-exact -- TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Written in the paper's own 1-based agent numbering and converted to 0-based
rows only in `peers`, so every line can be held against the text:

  tau, delta_r ..... Sec. 3.1, Eq. (2): bits of n-1, most significant first
  n_r .............. Sec. 3.1, Eq. (3): n_0 = 0, n_{r+1} = 2 n_r + delta_r
  2-port sender .... Sec. 3.1, Eqs. (5), (6): i receives from i - (n_r + delta_r)
  1-port partner ... Sec. 3.2, Eq. (7): odd i pairs with i + 2 n_r + 1, even i with i - 2 n_r - 1
  weights a, b ..... Algorithm 1 (Sec. 4.1)
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Tuple


def num_rounds(n: int) -> int:
    """tau = ceil(log2 n), taken as the bit length of n-1 (no floating point).  n = 1 -> 0."""
    if n < 1:
        raise ValueError("n must be >= 1")
    return (n - 1).bit_length()


def delta_bits(n: int) -> List[int]:
    """delta_0 .. delta_{tau-1}: the binary digits of n-1, delta_0 the most significant (Eq. 2)."""
    tau = num_rounds(n)
    return [((n - 1) >> (tau - 1 - r)) & 1 for r in range(tau)]


def window_sizes(n: int) -> List[int]:
    """n_0 .. n_tau with n_0 = 0 and n_{r+1} = 2 n_r + delta_r (Eq. 3); n_tau = n - 1."""
    nr = [0]
    for dlt in delta_bits(n):
        nr.append(2 * nr[-1] + dlt)
    return nr


def wrap(i: int, n: int) -> int:
    """The paper's index convention (Sec. 2.1, Notations): the representative of i in {1..n}."""
    return (i - 1) % n + 1


def sender(n: int, r: int, port: int, i: int) -> int:
    """1-based agent whose message agent i (1-based) receives in round r."""
    dlt = delta_bits(n)[r]
    m = window_sizes(n)[r]
    if port == 2:
        # Eq. (5) for delta_r = 1 (i - j = n_r + 1), Eq. (6) for delta_r = 0 (i - j = n_r)
        return wrap(i - (m + dlt), n)
    if port == 1:
        if n % 2:
            raise ValueError("CECA-1P is defined for even n only (Table 1, Sec. 3.2)")
        # Eq. (7)
        return wrap(i + 2 * m + 1, n) if i % 2 == 1 else wrap(i - 2 * m - 1, n)
    raise ValueError("port must be 1 or 2")


def peers(n: int, r: int, port: int) -> List[int]:
    """0-based receive-from map: row i takes the message of row peers[i]."""
    return [sender(n, r, port, i + 1) - 1 for i in range(n)]


def weights(n: int, r: int) -> Tuple[Fraction, Fraction]:
    """(a, b) of Algorithm 1: the self-weights of x and y in round r."""
    dlt = delta_bits(n)[r]
    m = window_sizes(n)[r]
    if dlt == 1:
        return Fraction(1, 2), Fraction(m, 2 * m + 1)
    return Fraction(m + 1, 2 * m + 1), Fraction(1, 2)


def exchanged(n: int, r: int) -> str:
    """Which variable travels in round r: "x" (the paper's I) when delta_r = 1, else "y" (J)."""
    return "x" if delta_bits(n)[r] == 1 else "y"
