"""The Python usage example of README.md runs as printed."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_readme_python_example_runs():
    print("case: README example", flush=True)
    text = open(os.path.join(ROOT, "README.md")).read()
    code = re.search(r"```python\n(.*?)```", text, flags=re.S).group(1)
    env = {}
    exec(compile(code, "README.md", "exec"), env)
    import torch
    torch.cuda.synchronize()
    assert len(env["w_local_0"]) == 3 and all(torch.isfinite(t).all() for t in env["w_local_0"])
    v = env["ctx"].ssd_get_state()
    assert v.iterations == 10 and v.local_updates == 8
    env["ctx"].close()
