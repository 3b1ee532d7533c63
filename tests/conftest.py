import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def load_paper_matrices():
    """Parse tests/golden/paper_matrices.txt -> {(algo, which, field): rows of Fraction}."""
    from fractions import Fraction
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_matrices.txt")
    out, key = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("@"):
            algo, which, field = line[1:].split("|")[0].split()
            key = (algo, which, field)
            out[key] = []
        else:
            out[key].append([Fraction(tok) for tok in line.split()])
    return out


@pytest.fixture(scope="session")
def paper_matrices():
    return load_paper_matrices()
