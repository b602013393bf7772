"""Per-agent stochastic gradients of the benchmark workloads, fp64 -- TEST INFRASTRUCTURE ONLY.

The paper asks only for one stochastic gradient per agent per iteration,
evaluated at z_i (Algorithm 1; problem statement Eq. (1)); its own least-squares
experiment (Sec. 5) uses f_i(x) = 1/2 ||A_i x - b_i||^2.  The minibatch forms
below belong to the benchmark configurations, not to the paper; the reading
taken is the *mean* over the B sampled rows (with the sum, the stated step size
diverges on the least-squares configuration).

Each factory returns grad(z, k) -> e with z, e of shape (n, d): row i is agent
i's gradient at its own z_i on its own minibatch of iteration k.
"""
from __future__ import annotations

import numpy as np

from . import noise


def lsq_loss_and_grad(Ab: np.ndarray, tb: np.ndarray, z: np.ndarray):
    """Minibatch least squares for one agent: F = 1/(2B) sum_j (a_j.z - t_j)^2 and its gradient."""
    res = Ab @ z - tb
    B = Ab.shape[0]
    return 0.5 * float(res @ res) / B, (Ab.T @ res) / B


def logistic_loss_and_grad(Ab: np.ndarray, lab: np.ndarray, z: np.ndarray):
    """Minibatch logistic loss, labels +-1: F = 1/B sum_j log(1 + exp(-y_j a_j.z)) and its gradient
    -1/B sum_j y_j sigma(-y_j a_j.z) a_j."""
    marg = lab * (Ab @ z)
    B = Ab.shape[0]
    loss = float(np.sum(np.logaddexp(0.0, -marg))) / B
    sig = np.exp(-np.logaddexp(0.0, marg))          # sigma(-marg), stable for both signs
    return loss, -(Ab.T @ (lab * sig)) / B


def make_minibatch_grad(kind: str, A: np.ndarray, t: np.ndarray, batch_idx: np.ndarray, k0: int = 0,
                        grad_scale: float = 0.0, noise_std: float = 0.0, seed: int = 0):
    """A (n, N, d), t (n, N) targets or labels, batch_idx (iters, n, B) rows drawn by the caller;
    iteration k uses batch_idx[(k - k0) mod iters].  grad_scale = 0 is the mean over the batch; grad_scale = s
    multiplies the *summed* gradient by s (s = 1 with the full batch is the gradient of 1/2 ||A_i x - b_i||^2,
    the local loss of the least-squares experiment, Sec. 5).  noise_std adds N(0, noise_std^2 I) drawn by
    oracle/noise.py, as that experiment does."""
    fn = {"lsq": lsq_loss_and_grad, "logistic": logistic_loss_and_grad}[kind]
    d = A.shape[2]
    cols = np.arange(d, dtype=np.int64)

    def grad(z: np.ndarray, k: int) -> np.ndarray:
        e = np.empty_like(z)
        for i in range(z.shape[0]):
            rows = batch_idx[(k - k0) % batch_idx.shape[0], i]
            Ab = A[i, rows].astype(np.float64)
            g = fn(Ab, t[i, rows].astype(np.float64), z[i])[1]          # mean over the B rows
            if grad_scale:
                g = g * (len(rows) * grad_scale)
            if noise_std:
                g = g + noise_std * noise.normals(seed, k, i, cols)
            e[i] = g
        return e

    return grad


def make_quad_center_grad(c: np.ndarray, noise_std: float, seed: int, columns=None):
    """e_i = z_i - c_i + noise_std * eps_i^(k): gradient of 1/2 ||z - c_i||^2 plus Gaussian noise drawn by
    the counter-based generator of oracle/noise.py.  `columns` gives the true column number of every
    column of c (for runs on a sampled subset of a wider problem); default 0..d-1."""
    n, d = c.shape
    cols = np.arange(d, dtype=np.int64) if columns is None else np.asarray(columns, dtype=np.int64)
    c64 = c.astype(np.float64)

    def grad(z: np.ndarray, k: int) -> np.ndarray:
        e = z - c64
        if noise_std != 0.0:
            for i in range(n):
                e[i] += noise_std * noise.normals(seed, k, i, cols)
        return e

    return grad
