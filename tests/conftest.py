import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line(
        "markers", "gpu: needs a real MI355X (run on the GPU box with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import spmm_oracle
    return spmm_oracle


# Largest relative error (|C_gpu - C_ref| / sum |a||b|) any GPU parity check of the run has
# seen; the terminal summary prints it so that a run's log holds the figure.
PARITY_WORST = {"err": 0.0}


def pytest_terminal_summary(terminalreporter):
    if PARITY_WORST["err"] > 0.0:
        terminalreporter.write_line("worst GPU parity error of this run: %.3e (bar 1e-5)" % PARITY_WORST["err"])
