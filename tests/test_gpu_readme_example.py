"""The usage example of README.md runs as written (GPU)."""
import os
import re

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_readme_usage_example_runs():
    import torch
    from gpu_helpers import load_product
    load_product()
    src = open(os.path.join(ROOT, "README.md")).read()
    code = re.search(r"```python\n(.*?)```", src, re.S).group(1)
    scope = {}
    exec(compile(code, "README.md", "exec"), scope)
    torch.cuda.synchronize()
    lay, views, shapes = scope["lay"], scope["views"], scope["shapes"]
    assert [tuple(v.shape) for v in views] == [tuple(s) for s in shapes]
    assert lay.padded == lay.shard * 8 and bool(torch.isfinite(scope["shards"][0]).all())
    assert float(scope["m"].abs().sum()) > 0.0            # the update ran
