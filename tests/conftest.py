import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    """The CPU oracle; built on demand (plain gcc, no GPU involved)."""
    from oracle import build as obuild
    from oracle import lq_ref
    if not os.path.exists(os.path.join(ROOT, "oracle", "liblq_oracle.so")):
        obuild.build()
    lq_ref.lib()
    return lq_ref
