"""The usage example in README.md runs as printed and does what the text around it says."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_readme_example_runs(gpu_lib):
    import torch
    text = open(os.path.join(ROOT, "README.md")).read()
    code = re.search(r"```python\n(.*?)```", text, re.S).group(1)
    ns = {}
    exec(compile(code, "README.md", "exec"), ns)
    torch.cuda.synchronize()
    d, acc, out, recv, bits = ns["d"], ns["acc"], ns["out"], ns["recv"], ns["bits"]
    a = acc.cpu().view(torch.int16).numpy().reshape(64, -1)
    o = out.cpu().view(torch.int16).numpy().reshape(64, -1)
    r = recv.cpu().view(torch.int16).numpy().reshape(64, -1)
    for k in range(64):                      # arrival k carried chunk seq[k]; 0 + x = x exactly
        s = int(d["seq"][k])
        zero_sign = (r[k] == np.int16(-32768))   # -0 + 0 = +0
        assert np.array_equal(a[s][~zero_sign], r[k][~zero_sign]) and np.array_equal(o[s], a[s])
    assert bits.cpu().numpy().view(np.uint32).tolist() == [0xFFFFFFFF, 0xFFFFFFFF]
