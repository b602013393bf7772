"""Pins for oracle/schedule.py: the paper's n = 6 example and structural facts (CPU only)."""
from fractions import Fraction

import pytest

from oracle import schedule as S


def test_n6_worked_example(golden):
    g = {ln.split()[0]: [int(v) for v in ln.split()[1:]] for ln in golden("ceca_n6_schedule.txt")}
    assert S.num_rounds(6) == g["tau"][0]
    assert S.delta_bits(6) == g["delta"]
    assert S.window_sizes(6) == g["n_r"]
    for r, s in enumerate(g["shift_2p"]):
        # agent i sends to i+s  <=>  i receives from i-s
        assert S.peers(6, r, 2) == [(i - s) % 6 for i in range(6)]


def test_n6_one_port_pairs(golden):
    for ln in golden("ceca_n6_pairs_1p.txt"):
        f = ln.split()
        r, delta, var = int(f[0]), int(f[1]), f[2]
        pairs = [tuple(int(v) for v in p.split("-")) for p in f[3:]]
        assert S.delta_bits(6)[r] == delta
        assert S.exchanged(6, r) == ("x" if var == "I" else "y")
        src = S.peers(6, r, 1)
        for a, b in pairs:
            assert src[a - 1] == b - 1 and src[b - 1] == a - 1


@pytest.mark.parametrize("n", list(range(1, 300)) + [1023, 1024, 1025, 4095, 4096, 4097])
def test_bits_and_windows(n):
    tau = S.num_rounds(n)
    # ceil(log2 n) without floating point
    assert (1 << tau) >= n and (tau == 0 or (1 << (tau - 1)) < n)
    d = S.delta_bits(n)
    assert len(d) == tau
    assert sum(b << (tau - 1 - r) for r, b in enumerate(d)) == n - 1
    if n >= 2:
        assert d[0] == 1
    nr = S.window_sizes(n)
    assert nr[0] == 0 and nr[-1] == n - 1      # "it is easy to verify that n_tau = n - 1"
    for r in range(tau):
        assert nr[r + 1] == 2 * nr[r] + d[r]


@pytest.mark.parametrize("n", list(range(2, 130)) + [1023, 1026])
def test_two_port_is_cyclic_shift(n):
    for r in range(S.num_rounds(n)):
        s = S.window_sizes(n)[r] + S.delta_bits(n)[r]
        src = S.peers(n, r, 2)
        assert sorted(src) == list(range(n))
        assert all(src[i] == (i - s) % n for i in range(n))
        assert 1 <= s <= n - 1


@pytest.mark.parametrize("n", list(range(2, 202, 2)) + [1026, 4096])
def test_one_port_is_perfect_matching(n):
    for r in range(S.num_rounds(n)):
        src = S.peers(n, r, 1)
        assert sorted(src) == list(range(n))
        assert all(src[src[i]] == i and src[i] != i for i in range(n))
        # partners have opposite parity
        assert all((src[i] - i) % 2 == 1 for i in range(n))


@pytest.mark.parametrize("n", [3, 5, 7, 31, 101])
def test_one_port_rejects_odd_n(n):
    with pytest.raises(ValueError):
        S.peers(n, 0, 1)


def test_weights_table():
    # Algorithm 1: delta = 1 -> a = 1/2, b = n_r/(2 n_r + 1);  delta = 0 -> a = (n_r+1)/(2 n_r+1), b = 1/2
    F = Fraction
    assert [S.weights(6, r) for r in range(3)] == [(F(1, 2), F(0)), (F(2, 3), F(1, 2)), (F(1, 2), F(2, 5))]
    assert [S.weights(5, r) for r in range(3)] == [(F(1, 2), F(0)), (F(2, 3), F(1, 2)), (F(3, 5), F(1, 2))]
    for n in range(2, 200):
        for r in range(S.num_rounds(n)):
            a, b = S.weights(n, r)
            m = S.window_sizes(n)[r]
            # weights are the window-size ratios that keep Eq. (4) true
            if S.delta_bits(n)[r]:
                assert a == F(m + 1, 2 * m + 2) and b == F(m, 2 * m + 1)
            else:
                assert a == F(m + 1, 2 * m + 1) and b == F(m, 2 * m)


def test_config_sizes():
    assert S.delta_bits(100) == [1, 1, 0, 0, 0, 1, 1]
    assert S.window_sizes(100) == [0, 1, 3, 6, 12, 24, 49, 99]
    assert S.delta_bits(31) == [1, 1, 1, 1, 0]
    assert S.window_sizes(31) == [0, 1, 3, 7, 15, 30]
    assert S.delta_bits(1023) == [1] * 9 + [0]
