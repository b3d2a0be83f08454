import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# tests/test_oracle_mutants.py runs the pin tests against a deliberately broken copy of the oracle package
if os.environ.get("MW_ORACLE_UNDER_TEST"):
    sys.path.insert(0, os.environ["MW_ORACLE_UNDER_TEST"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden(name):
    return os.path.join(ROOT, "tests", "golden", name)


@pytest.fixture(scope="session")
def host_pools():
    from workloads import HostPools

    return HostPools()
