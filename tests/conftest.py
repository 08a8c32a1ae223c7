import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# test_oracle_mutations.py runs the pins against deliberately broken copies of the oracle:
# the directory named here (holding oracle/lagkv_oracle.py) then shadows the real package
if os.environ.get("LAGKV_ORACLE_OVERRIDE"):
    sys.path.insert(0, os.environ["LAGKV_ORACLE_OVERRIDE"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
