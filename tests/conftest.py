import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU parity runs use the oracle as built from oracle/step.c and nothing else: the
    switch that lets the mutant tests load a deliberately broken oracle must be off."""
    if os.environ.get("PS_ORACLE_LIB_UNDER_TEST") and any(i.get_closest_marker("gpu") for i in items):
        raise pytest.UsageError("PS_ORACLE_LIB_UNDER_TEST is set: GPU tests would be checked "
                                "against a substituted oracle; unset it")


def load_golden(name="paper_values.txt"):
    """Parse ``key = value  # citation`` lines of a golden fixture into a dict of str."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


@pytest.fixture(scope="session")
def golden():
    return load_golden()
