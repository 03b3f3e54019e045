import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def read_golden(name):
    """Parse a 'key: v1 v2 ...' fixture; values may be integers or p/q fractions."""
    from fractions import Fraction
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key.strip()] = [float(Fraction(v)) for v in vals.split()]
    return out


@pytest.fixture(scope="session")
def oracle():
    from oracle import laplex_oracle
    laplex_oracle.build()
    return laplex_oracle
