import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden(name):
    """Parse a tests/golden text fixture: '#' comments, whitespace separated tokens per line."""
    rows = []
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def fw():
    """The GPU library binding; GPU tests fail loudly if it cannot be loaded."""
    import torch
    assert torch.cuda.is_available(), "GPU test collected on a machine without a GPU"
    from paper_2010_01546_amd import binding
    return binding
