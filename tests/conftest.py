import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # A GPU test on a box without a GPU is an error of the run, not a skip:
    # the HIP path must be the one that executes.  Nothing to do here except
    # keep CPU-only runs (-m "not gpu") free of any device initialisation.
    return
