"""Consensus observables, fp64 -- TEST INFRASTRUCTURE ONLY.

  mean ............ x_bar = (1/n) sum_i x_i                     (Sec. 4.2, before Theorem 4.3)
  frob2 ........... ||x - 1 x_bar^T||_F^2                       (descent lemma, App. B.3)
  residue ......... sum_i ||x_i - x_bar||                       (Sec. 5, finite-time consensus experiment)
  max_dev ......... max_i ||x_i - x_bar||
  mean_norm ....... ||x_bar||
"""
from __future__ import annotations

import numpy as np


def consensus_error(x: np.ndarray):
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    xbar = x.sum(axis=0) / n
    dev = np.sqrt(((x - xbar) ** 2).sum(axis=1))
    return {
        "frob2": float((dev ** 2).sum()),
        "residue": float(dev.sum()),
        "max_dev": float(dev.max()),
        "mean_norm": float(np.sqrt((xbar ** 2).sum())),
        "mean": xbar,
    }
