import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' comments, '[tag] rows cols' blocks of numbers."""
    import numpy as np
    path = os.path.join(ROOT, "tests", "golden", name)
    out, tag, shape, buf = {}, None, None, []

    def flush():
        if tag is not None:
            out[tag] = np.array(buf, dtype=np.float64).reshape(shape)

    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("["):
                flush()
                head, dims = line[1:].split("]")
                tag, shape, buf = head.strip(), tuple(int(d) for d in dims.split()), []
            else:
                buf.extend(float(t) for t in line.split())
    flush()
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden
