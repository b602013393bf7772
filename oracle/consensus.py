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


def state_consensus(x: np.ndarray, y: np.ndarray):
    """Consensus observables of the stacked state: those of x, those of y (each about its own mean),
    and ||phi||_F^2 = ||x - 1 x_bar^T||_F^2 + ||y - 1 y_bar^T||_F^2, the quantity the consensus lemma
    bounds (App. B.3, definition of phi before the consensus lemma)."""
    cx = consensus_error(x)
    cy = consensus_error(y)
    return {"x": cx, "y": cy, "phi2": cx["frob2"] + cy["frob2"]}
