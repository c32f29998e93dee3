import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# tests/test_oracle_mutations.py re-runs the oracle's pins in child processes against copies of the oracle with a
# mistake planted in them; the copy's parent directory comes first on the path there.
if os.environ.get("MOEP_TEST_ORACLE_ROOT"):
    sys.path.insert(0, os.environ["MOEP_TEST_ORACLE_ROOT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
