import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import nqkv_oracle
    nqkv_oracle.build()
    return nqkv_oracle


def load_golden(filename: str) -> dict:
    """tests/golden/<filename>: 'name = v [v ...]' lines ('#' comments) -> {name: float | [float, ...]}."""
    out = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", filename)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            name, val = (t.strip() for t in line.split("=", 1))
            nums = [float(v) for v in val.split()]
            out[name] = nums[0] if len(nums) == 1 else nums
    return out
