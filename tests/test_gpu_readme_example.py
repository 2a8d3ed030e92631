"""The usage example printed in README.md runs as written."""
import os
import re

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_readme_python_example_runs():
    torch = pytest.importorskip("torch")
    path = os.path.join(ROOT, "README.md")
    if not os.path.exists(path):
        pytest.skip("README.md is not part of this copy of the tree")
    text = open(path).read()
    blocks = re.findall(r"```python\n(.*?)```", text, flags=re.S)
    assert len(blocks) == 1
    scope = {}
    exec(compile(blocks[0], "README.md", "exec"), scope)
    torch.cuda.synchronize()
    sc = scope["scalars"].cpu()
    assert sc[0].item() == 0.0 and sc[3:4].view(torch.int32).item() == 0        # zero gradients: norm 0, no flag
    # p = 0 and g = 0: the step leaves the state at zero and writes zeros to the working copy
    assert not scope["state"].any().item() and not scope["params16"].view(torch.int16).any().item()
