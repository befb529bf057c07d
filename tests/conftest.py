import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse tests/golden/<name>: '#' comment lines, 'key = v1 v2 ...' value lines."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, val = line.split("=", 1)
            out[key.strip()] = [float(v) for v in val.split()]
    return out


@pytest.fixture(scope="session")
def orc():
    from oracle import aweq_oracle
    aweq_oracle.lib()
    return aweq_oracle


def from_panels(buf, rows, K):
    """Row-major [rows, K] view of an int8 buffer in the library's K-panel layout (panel p =
    columns 64 p .. 64 p + 63 of every row, rows back to back); checks the zero fill past K."""
    import numpy as np
    kp = -(-K // 64)
    a = np.asarray(buf).reshape(-1)
    assert a.size >= kp * rows * 64
    a = a[:kp * rows * 64].reshape(kp, rows, 64).transpose(1, 0, 2).reshape(rows, kp * 64)
    assert not a[:, K:].any(), "columns past K must be zero"
    return np.ascontiguousarray(a[:, :K])


def to_panels(mat):
    """K-panel layout (flat) of a row-major int8 matrix."""
    import numpy as np
    rows, K = mat.shape
    kp = -(-K // 64)
    padded = np.zeros((rows, kp * 64), dtype=mat.dtype)
    padded[:, :K] = mat
    return np.ascontiguousarray(padded.reshape(rows, kp, 64).transpose(1, 0, 2)).reshape(-1)
