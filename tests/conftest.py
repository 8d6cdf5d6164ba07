import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--oracle-lib", default=None,
                     help="run against this build of the oracle library (used by the mutation test only)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle(request):
    from oracle import agent_attn_oracle
    alt = request.config.getoption("--oracle-lib")
    if alt:
        agent_attn_oracle.use_library(alt)
    else:
        agent_attn_oracle.build()
    return agent_attn_oracle
