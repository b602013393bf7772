"""The usage example printed in README.md runs as written and ends with every agent at the same model."""
import os
import re

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_readme_example_runs():
    import torch
    text = open(os.path.join(ROOT, "README.md")).read()
    code = re.search(r"```python\n(.*?)```", text, flags=re.S).group(1)
    target = torch.linspace(-1.0, 1.0, 4096, device="cuda")

    def my_loss(z):
        shift = torch.arange(z.shape[0], device="cuda", dtype=torch.float32)[:, None]      # every agent its own optimum
        return 0.5 * ((z - target - 0.1 * shift) ** 2).sum()

    scope = {"my_loss": my_loss}
    exec(compile(code, "README.md", "exec"), scope)
    torch.cuda.synchronize()
    S, n = scope["S"], scope["n"]
    x, y = S[:n], S[n:]
    assert torch.isfinite(S).all()
    assert (x - x[0]).abs().max().item() <= 1e-6 and (y - x[0]).abs().max().item() <= 1e-6
    # 100 iterations at step 0.1 bring the average close to the average optimum (1 - 0.9^100 of the way)
    want = target + 0.1 * (n - 1) / 2
    assert (x[0] - want).abs().max().item() <= 1e-3
