"""Seeded synthetic inputs for the DSGD-CECA hot path.

This module only *draws data*: it holds none of the method's arithmetic (no
schedule, no gossip weights, no gradients) and imports neither the oracle nor
the HIP binding, so both sides can be fed the very same arrays.

The five workloads mirror the shapes of the paper's least-squares experiment
(Sec. 5, "DSGD: least-squares problem": A_i ~ N(0, I), b_i = A_i x* + v_i) and
of a flat deep-network parameter vector; they stand in for the MNIST / CIFAR-10
runs of Sec. 5 and App. D, whose datasets are not available here.  Every
generator takes explicit sizes so tests can shrink a workload while keeping its
structure.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    """Sizes and hyper-parameters of one workload (nothing is drawn here)."""

    name: str
    n: int            # agents at the stated port
    port: int         # 1 or 2
    d: int            # parameters per agent
    loss: str         # "lsq" | "logistic" | "quad_center" | "none"
    N: int = 0        # samples per agent
    B: int = 0        # minibatch rows per agent per iteration
    lr: float = 0.0
    iters: int = 0
    seed: int = 0
    noise_std: float = 0.0     # additive Gaussian gradient noise
    grad_scale: float = 0.0    # minibatch losses: 0 = mean over the batch, s = factor on the summed gradient
    obs_noise: float = 0.1     # least squares: standard deviation of the measurement noise in b
    lr_decay: float = 1.0      # step size is lr / lr_decay^(k // lr_decay_every)
    lr_decay_every: int = 0


# The five configurations.  CECA-1P exists for even n only (Table 1), so the two
# configurations that ask for 1P at an odd n are carried twice: 2P at the stated
# n and 1P at the nearest even n with the same number of rounds.
SPECS = {
    "lsq5_2p": WorkloadSpec("lsq5_2p", n=5, port=2, d=1000, loss="lsq", N=64, B=8, lr=0.01, iters=200, seed=0),
    "lsq6_1p": WorkloadSpec("lsq6_1p", n=6, port=1, d=1000, loss="lsq", N=64, B=8, lr=0.01, iters=200, seed=0),
    "logistic6_2p": WorkloadSpec("logistic6_2p", n=6, port=2, d=10_000, loss="logistic", N=2000, B=32,
                                 lr=0.05, iters=500, seed=1),
    "gossip100_1p": WorkloadSpec("gossip100_1p", n=100, port=1, d=1 << 20, loss="none", seed=2),
    "gossip100_2p": WorkloadSpec("gossip100_2p", n=100, port=2, d=1 << 20, loss="none", seed=2),
    "quad31_2p": WorkloadSpec("quad31_2p", n=31, port=2, d=25_557_032, loss="quad_center", lr=0.1, iters=50,
                              seed=3, noise_std=0.01),
    "quad30_1p": WorkloadSpec("quad30_1p", n=30, port=1, d=25_557_032, loss="quad_center", lr=0.1, iters=50,
                              seed=3, noise_std=0.01),
    # the paper's own least-squares experiment (Sec. 5): full gradient of 1/2 ||A_i x - b_i||^2 plus N(0, 25 I)
    # noise, n = 258 agents, d = 10, N = 50, step 0.02 divided by 1.5 every 20 iterations
    "paperlsq258_1p": WorkloadSpec("paperlsq258_1p", n=258, port=1, d=10, loss="lsq", N=50, B=50, lr=0.02, iters=200,
                                   seed=5, noise_std=5.0, grad_scale=1.0, obs_noise=0.1, lr_decay=1.5,
                                   lr_decay_every=20),
    "paperlsq258_2p": WorkloadSpec("paperlsq258_2p", n=258, port=2, d=10, loss="lsq", N=50, B=50, lr=0.02, iters=200,
                                   seed=5, noise_std=5.0, grad_scale=1.0, obs_noise=0.1, lr_decay=1.5,
                                   lr_decay_every=20),
    "logistic1023_2p": WorkloadSpec("logistic1023_2p", n=1023, port=2, d=4096, loss="logistic", N=512, B=16,
                                    lr=0.02, iters=2000, seed=4),
}


def step_size(spec: WorkloadSpec, k: int) -> float:
    """Step size of iteration k under the workload's decay schedule."""
    if spec.lr_decay_every:
        return spec.lr / spec.lr_decay ** (k // spec.lr_decay_every)
    return spec.lr


def for_run(spec: WorkloadSpec, run: int) -> WorkloadSpec:
    """The same workload with the seed of independent run number `run` (run 0 is the workload itself): the
    paper averages its least-squares experiment over five runs and its consensus comparison over three
    (Sec. 5)."""
    return dataclasses.replace(spec, seed=spec.seed + 7919 * run)


def full_batch_indices(n: int, N: int) -> np.ndarray:
    """Every agent uses all of its N rows: shape (1, n, N) int32 (one entry serves every iteration)."""
    return np.tile(np.arange(N, dtype=np.int32), (1, n, 1))


def shrink(spec: WorkloadSpec, **kw) -> WorkloadSpec:
    """The same workload at other sizes (used by tests)."""
    return dataclasses.replace(spec, **kw)


def _rng(seed: int, stream: int) -> np.random.Generator:
    # independent child streams so that shrinking one array does not shift another
    return np.random.default_rng(np.random.SeedSequence([seed, stream]))


def initial_state(n: int, d: int, seed: int, kind: str = "normal") -> np.ndarray:
    """x(0), shape (n, d) float32.  kind = "normal" (N(0,1) entries) or "zero"."""
    if kind == "zero":
        return np.zeros((n, d), dtype=np.float32)
    return _rng(seed, 0).standard_normal((n, d), dtype=np.float32)


def batch_indices(n: int, N: int, B: int, iters: int, seed: int) -> np.ndarray:
    """Minibatch row numbers, shape (iters, n, B) int32, uniform on [0, N) with replacement."""
    return _rng(seed, 1).integers(0, N, size=(iters, n, B), dtype=np.int32)


def lsq_data(n: int, N: int, d: int, seed: int, obs_noise: float = 0.1):
    """Least-squares data: A (n, N, d), b (n, N), x_star (d,), all float32."""
    g = _rng(seed, 2)
    A = g.standard_normal((n, N, d), dtype=np.float32)
    x_star = g.standard_normal(d, dtype=np.float32)
    v = g.standard_normal((n, N), dtype=np.float32)
    b = (A.astype(np.float64) @ x_star.astype(np.float64) + obs_noise * v).astype(np.float32)
    return A, b, x_star


def logistic_data_hetero(n: int, N: int, d: int, seed: int, mu_std: float = 0.5, label_noise: float = 0.1):
    """Non-iid logistic data: features N(mu_i, I) with mu_i ~ N(0, mu_std^2 I) per agent,
    labels sign(a.w* + label_noise*N(0,1)) in {-1,+1} (0 maps to +1).  Returns A (n,N,d), labels (n,N), w_star."""
    g = _rng(seed, 3)
    w_star = g.standard_normal(d, dtype=np.float32)
    A = np.empty((n, N, d), dtype=np.float32)
    lab = np.empty((n, N), dtype=np.float32)
    for i in range(n):
        mu = (mu_std * g.standard_normal(d)).astype(np.float32)
        A[i] = g.standard_normal((N, d), dtype=np.float32) + mu
        s = A[i].astype(np.float64) @ w_star.astype(np.float64) + label_noise * g.standard_normal(N)
        lab[i] = np.where(s >= 0, 1.0, -1.0)
    return A, lab, w_star


def logistic_data_sparse(n: int, N: int, d: int, seed: int, density: float = 0.1, flip: float = 0.05):
    """Logistic data with N(0,1) features of which a `density` fraction is non-zero (dense storage),
    labels sign(a.w*) with a `flip` fraction inverted.  Returns A (n,N,d), labels (n,N), w_star."""
    g = _rng(seed, 4)
    w_star = g.standard_normal(d, dtype=np.float32)
    A = np.empty((n, N, d), dtype=np.float32)
    lab = np.empty((n, N), dtype=np.float32)
    for i in range(n):
        Ai = g.standard_normal((N, d), dtype=np.float32)
        Ai *= (g.random((N, d), dtype=np.float32) < density)
        A[i] = Ai
        s = Ai.astype(np.float64) @ w_star.astype(np.float64)
        y = np.where(s >= 0, 1.0, -1.0)
        y[g.random(N) < flip] *= -1.0
        lab[i] = y
    return A, lab, w_star


def quad_centers(n: int, d: int, seed: int) -> np.ndarray:
    """Per-agent centres c_i ~ N(0,1)^d of the quadratic loss, shape (n, d) float32."""
    return _rng(seed, 5).standard_normal((n, d), dtype=np.float32)


# ---------------------------------------------------------------------------
# Device-side generation for the workloads that are too large to draw on the
# host in reasonable time (n*d ~ 8e8).  torch is only a random-number source
# and an allocator here.
# ---------------------------------------------------------------------------

def device_normal(shape, seed: int, device: str = "cuda", out=None):
    """N(0,1) float32 tensor drawn on `device` from a seeded torch generator."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=device)
    # row by row keeps the transient memory of the generator small for multi-GB tensors
    if out.dim() >= 2:
        for i in range(out.shape[0]):
            out[i].normal_(generator=gen)
    else:
        out.normal_(generator=gen)
    return out


def device_logistic_sparse(n: int, N: int, d: int, seed: int, device: str = "cuda",
                           density: float = 0.1, flip: float = 0.05):
    """Device version of `logistic_data_sparse` (same structure, torch generator)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    w_star = torch.empty(d, dtype=torch.float32, device=device).normal_(generator=gen)
    w64 = w_star.double()
    A = torch.empty((n, N, d), dtype=torch.float32, device=device)
    lab = torch.empty((n, N), dtype=torch.float32, device=device)
    for i in range(n):
        Ai = A[i]
        Ai.normal_(generator=gen)
        mask = torch.empty((N, d), dtype=torch.float32, device=device).uniform_(generator=gen) < density
        Ai.mul_(mask)
        # elementwise product and row sums in fp64: no matrix-product library is pulled in just to draw labels
        s = (Ai.double() * w64).sum(dim=1)
        y = torch.where(s >= 0, 1.0, -1.0).float()
        fl = torch.empty(N, dtype=torch.float32, device=device).uniform_(generator=gen) < flip
        lab[i] = torch.where(fl, -y, y)
    return A, lab, w_star


def sample_columns(d: int, count: int, seed: int, tile: int = 1024, tail: Optional[int] = None) -> np.ndarray:
    """Sorted column numbers for sampled full-size parity: the first and last `tile` boundary
    neighbourhoods, the ragged tail, and uniformly drawn columns in between."""
    g = _rng(seed, 6)
    cols = set()
    edge = [0, 1, 2, 3, tile - 1, tile, tile + 1, d - 1, d - 2, d - 3, d - 4, d - 5, (d // tile) * tile,
            max((d // tile) * tile - 1, 0), d // 2, d // 2 + 1]
    for c in edge:
        if 0 <= c < d:
            cols.add(int(c))
    if tail:
        for c in range(max(d - tail, 0), d):
            cols.add(c)
    need = max(count - len(cols), 0)
    if need:
        for c in g.integers(0, d, size=need):
            cols.add(int(c))
    return np.array(sorted(cols), dtype=np.int64)


# ---------------------------------------------------------------------------------------------
# Graph tables for ceca_graph_rounds: neighbour lists of standard graphs with Metropolis weights
# (inputs only: which vertices are adjacent and the textbook weight 1 / (1 + max degree of the two ends))
# ---------------------------------------------------------------------------------------------
def graph_table(n: int, edges, m: int = 0):
    """(nbr (n, m) int32, w (n, m) float32, w_self (n,) float32) of the undirected graph with Metropolis
    weights; rows with fewer neighbours are padded with the vertex itself at weight 0."""
    adj = [[] for _ in range(n)]
    for a, b in edges:
        if a != b and b not in adj[a]:
            adj[a].append(b)
            adj[b].append(a)
    width = max(m, max(len(r) for r in adj), 1)
    nbr = np.tile(np.arange(n, dtype=np.int32)[:, None], (1, width))
    w = np.zeros((n, width), dtype=np.float32)
    for i in range(n):
        for j, v in enumerate(sorted(adj[i])):
            nbr[i, j] = v
            w[i, j] = np.float32(1.0 / (1.0 + max(len(adj[i]), len(adj[v]))))
    w_self = (1.0 - w.astype(np.float64).sum(axis=1)).astype(np.float32)
    return nbr, w, w_self


def edges_of(kind: str, n: int, rows: int = 0):
    """Edge lists: 'ring', 'hypercube' (n a power of two), 'torus' / 'grid' (rows x n/rows), 'random' (ring plus n chords)."""
    if kind == "ring":
        return [(i, (i + 1) % n) for i in range(n)]
    if kind == "hypercube":
        return [(i, i ^ (1 << b)) for i in range(n) for b in range(max(n - 1, 1).bit_length()) if (i ^ (1 << b)) < n and i < (i ^ (1 << b))]
    if kind in ("torus", "grid"):
        cols = n // rows
        e = []
        for a in range(rows):
            for b in range(cols):
                if kind == "torus" or a + 1 < rows:
                    e.append((a * cols + b, ((a + 1) % rows) * cols + b))
                if kind == "torus" or b + 1 < cols:
                    e.append((a * cols + b, a * cols + (b + 1) % cols))
        return e
    if kind == "random":
        rng = np.random.default_rng(n)
        chords = [(int(a), int(b)) for a, b in rng.integers(0, n, size=(n, 2)) if a != b]
        return [(i, (i + 1) % n) for i in range(n)] + chords
    raise ValueError(kind)
