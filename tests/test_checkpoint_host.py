"""Checkpoint file round trip on the CPU (no library call involved)."""
import numpy as np
import pytest
import torch

from paper_2306_00256_amd import checkpoint as CK


def test_round_trip_keeps_bits_and_strips_padding(tmp_path):
    n, d, ld = 5, 37, 48
    rng = np.random.default_rng(0)
    S = torch.from_numpy(rng.standard_normal((2 * n, ld)).astype(np.float32))
    S[3, 7] = float("inf")
    S[4, 0] = -0.0
    p = str(tmp_path / "s.ckpt")
    CK.save_state(p, S, n, d, k=123, meta={"workload": "toy", "port": 2})
    T, n2, d2, k2, meta = CK.load_state(p, device="cpu", ld=64)
    assert (n2, d2, k2) == (n, d, 123) and meta == {"workload": "toy", "port": 2}
    assert T.shape == (2 * n, 64) and torch.all(T[:, d:] == 0)
    assert np.array_equal(T[:, :d].numpy().view(np.uint32), S[:, :d].numpy().view(np.uint32))
    CK.save_state(p, T, n, d, k=124)                                  # overwrite in place
    assert CK.load_state(p, device="cpu")[3] == 124


def test_rejects_damaged_files(tmp_path):
    p = str(tmp_path / "s.ckpt")
    S = torch.zeros((4, 8), dtype=torch.float32)
    CK.save_state(p, S, 2, 8, 0)
    raw = open(p, "rb").read()
    open(p, "wb").write(raw[:-4])
    with pytest.raises(ValueError):
        CK.load_state(p, device="cpu")
    open(p, "wb").write(b'{"magic": "other"}\n')
    with pytest.raises(ValueError):
        CK.load_state(p, device="cpu")
    with pytest.raises(ValueError):
        CK.save_state(p, S.double(), 2, 8, 0)
    with pytest.raises(ValueError):
        CK.save_state(p, S, 3, 8, 0)
