import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_paper_constants():
    path = os.path.join(ROOT, "tests", "golden", "paper_constants.txt")
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = [s.strip() for s in line.split("=", 1)]
            vals = [float(x) for x in v.split()]
            out[k] = vals if len(vals) > 1 else vals[0]
    return out


@pytest.fixture(scope="session")
def paper_constants():
    return load_paper_constants()


# A planted mistake for tests/test_oracle_mutations.py (applied to the oracle on the CPU only).
if os.environ.get("ORACLE_MUTATION"):
    from oracle import lopt_oracle as _O
    from tests.oracle_mutations import MUTATIONS as _M
    _M[os.environ["ORACLE_MUTATION"]](_O)
