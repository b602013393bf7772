"""Checkpoint of a DSGD-CECA run: the stacked state S = [x; y] and the iteration counter k.

Algorithm 1's whole state is (x, y, k): the round index is k mod tau, and every random draw of this
library is a function of (seed, k, agent, column), so a run resumed from a checkpoint continues with
exactly the bits it would have had.  File layout: one ASCII line of JSON (magic, n, d, k, user
metadata) ending in a newline, then 2n*d little-endian fp32 values, row-major, without row padding.
"""
from __future__ import annotations

import json
import os
from typing import Optional, Tuple

import numpy as np
import torch

MAGIC = "dsgd-ceca-state-1"


def save_state(path: str, S: torch.Tensor, n: int, d: int, k: int, meta: Optional[dict] = None) -> None:
    """Write rows 0..2n-1, columns 0..d-1 of S (any device, any row pitch) and k; replaces `path` atomically."""
    if S.dtype != torch.float32 or S.dim() != 2 or S.shape[0] < 2 * n or S.shape[1] < d:
        raise ValueError("S must be a float32 matrix with at least 2n rows and d columns")
    host = S[: 2 * n, :d].detach().to("cpu").contiguous().numpy()
    header = json.dumps({"magic": MAGIC, "n": int(n), "d": int(d), "k": int(k), "meta": meta or {}})
    tmp = path + ".tmp"
    with open(tmp, "wb") as f:
        f.write(header.encode("ascii") + b"\n")
        host.astype("<f4", copy=False).tofile(f)
        f.flush()
        os.fsync(f.fileno())
    os.replace(tmp, path)


def load_state(path: str, device="cuda", ld: Optional[int] = None) -> Tuple[torch.Tensor, int, int, int, dict]:
    """Returns (S, n, d, k, meta); S is a fresh 2n x ld float32 tensor on `device` (ld defaults to d,
    padding columns are zero)."""
    with open(path, "rb") as f:
        head = json.loads(f.readline().decode("ascii"))
        if head.get("magic") != MAGIC:
            raise ValueError(f"{path}: not a DSGD-CECA state file")
        n, d, k = int(head["n"]), int(head["d"]), int(head["k"])
        data = np.fromfile(f, dtype="<f4")
    if n < 1 or d < 1 or k < 0 or data.size != 2 * n * d:
        raise ValueError(f"{path}: header says n={n}, d={d}, k={k} but the file holds {data.size} values")
    ld = d if ld is None else int(ld)
    if ld < d:
        raise ValueError("ld < d")
    S = torch.zeros((2 * n, ld), dtype=torch.float32, device=device)
    S[:, :d] = torch.from_numpy(data.reshape(2 * n, d).astype(np.float32, copy=False)).to(device)
    return S, n, d, k, head.get("meta", {})
