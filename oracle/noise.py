"""Counter-based Gaussian noise for the quadratic-centre workload -- TEST INFRASTRUCTURE ONLY.

The paper's least-squares experiment (Sec. 5) adds N(0, sigma^2 I) noise to each
agent's gradient but names no generator; the generator below is this build's own
definition (parity with the paper is therefore unpinned for the stream itself;
tests pin only its distribution).  The integer part is specified exactly so a
device implementation can reproduce it bit for bit:

  mix(h):     h ^= h >> 16;  h *= 0x7feb352d;  h ^= h >> 15;  h *= 0x846ca68b;  h ^= h >> 16     (uint32)
  keys:       k0 = mix( mix(seed + 0x9e3779b9 * k) ^ agent );   k1 = mix(k0 + 0x85ebca6b)
  word(c):    h = c ^ k0;  h ^= h >> 16;  h *= 0x7feb352d;  h ^= h >> 15;  h += k1;
              h *= 0x846ca68b;  h ^= h >> 16
  pair q = column >> 1:   w1 = word(2q), w2 = word(2q + 1)
              u1 = ((w1 >> 8) + 1) / 2^24  in (0, 1],     u2 = (w2 >> 8) / 2^24  in [0, 1)
  Box-Muller: rad = sqrt(-2 ln u1);  eps[2q] = rad * cos(2 pi u2),  eps[2q+1] = rad * sin(2 pi u2)

(k is the iteration, agent the 0-based row the gradient belongs to, column the 0-based parameter.)
"""
from __future__ import annotations

import numpy as np

_M1 = np.uint32(0x7FEB352D)
_M2 = np.uint32(0x846CA68B)


def _mix(h: np.ndarray) -> np.ndarray:
    h = h.astype(np.uint32)
    h = h ^ (h >> np.uint32(16))
    h = h * _M1
    h = h ^ (h >> np.uint32(15))
    h = h * _M2
    h = h ^ (h >> np.uint32(16))
    return h


def stream_keys(seed: int, k: int, agent: int):
    with np.errstate(over="ignore"):
        s = np.uint32(seed & 0xFFFFFFFF) + np.uint32(0x9E3779B9) * np.uint32(k & 0xFFFFFFFF)
        k0 = _mix(_mix(np.array(s)) ^ np.uint32(agent))
        k1 = _mix(k0 + np.uint32(0x85EBCA6B))
    return k0, k1


def _word(c: np.ndarray, k0, k1) -> np.ndarray:
    with np.errstate(over="ignore"):
        h = c.astype(np.uint32) ^ k0
        h = h ^ (h >> np.uint32(16))
        h = h * _M1
        h = h ^ (h >> np.uint32(15))
        h = h + k1
        h = h * _M2
        h = h ^ (h >> np.uint32(16))
    return h


def normals(seed: int, k: int, agent: int, columns: np.ndarray) -> np.ndarray:
    """eps(seed, k, agent, column) for an array of 0-based columns, float64."""
    columns = np.asarray(columns, dtype=np.int64)
    k0, k1 = stream_keys(seed, k, agent)
    q = (columns >> 1).astype(np.uint32)
    with np.errstate(over="ignore"):
        w1 = _word(q * np.uint32(2), k0, k1)
        w2 = _word(q * np.uint32(2) + np.uint32(1), k0, k1)
    u1 = ((w1 >> np.uint32(8)).astype(np.float64) + 1.0) / 16777216.0
    u2 = (w2 >> np.uint32(8)).astype(np.float64) / 16777216.0
    rad = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    return np.where(columns & 1, rad * np.sin(ang), rad * np.cos(ang))
