"""Helpers shared by the GPU parity tests (argument plumbing and error measures only)."""
import numpy as np


def rel_err(got: np.ndarray, want: np.ndarray):
    """(max-norm relative error, Frobenius relative error) over a whole state."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den_m = max(np.abs(want).max(), 1e-300)
    den_f = max(np.sqrt((want ** 2).sum()), 1e-300)
    return np.abs(got - want).max() / den_m, np.sqrt(((got - want) ** 2).sum()) / den_f


def make_state(torch, x0: np.ndarray, y0=None, ld=None, pad_value=12345.0, offset=0):
    """Device state of 2n rows of ld floats from x0 (n, d); padding columns hold `pad_value`.
    `offset` shifts the base pointer by that many floats (to reach the unaligned kernels)."""
    n, d = x0.shape
    ld = d if ld is None else ld
    flat = torch.full((2 * n * ld + offset,), pad_value, dtype=torch.float32, device="cuda")
    S = flat[offset:].view(2 * n, ld)
    S[:n, :d] = torch.from_numpy(np.ascontiguousarray(x0, dtype=np.float32)).cuda()
    S[n:, :d] = torch.from_numpy(np.ascontiguousarray(x0 if y0 is None else y0, dtype=np.float32)).cuda()
    return S


def split_state(S, n, d):
    h = S.cpu().numpy()
    return h[:n, :d].astype(np.float64), h[n:, :d].astype(np.float64)
