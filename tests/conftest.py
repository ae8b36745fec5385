import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C-ABI HIP library)")


def load_table1():
    """Parse tests/golden/table1_flops.txt -> {name: callable(n,i,o,r)}."""
    path = os.path.join(ROOT, "tests", "golden", "table1_flops.txt")
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, expr = [s.strip() for s in line.split(":", 1)]
            code = compile(expr, name, "eval")
            out[name] = (lambda c: (lambda n, i, o, r: eval(c, {"__builtins__": {}}, dict(n=n, i=i, o=o, r=r))))(code)
    return out


@pytest.fixture(scope="session")
def table1():
    return load_table1()
