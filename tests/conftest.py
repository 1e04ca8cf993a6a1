import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden_path(name):
    return os.path.join(ROOT, "tests", "golden", name)


@pytest.fixture(scope="session")
def partition_golden():
    keys, perms = [], []
    with open(golden_path("partition_vectors.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "key":
                keys.append((int(tok[1]), int(tok[2]), int(tok[3], 16)))
            elif tok[0] == "perm":
                seed, t, W = int(tok[1]), int(tok[2]), int(tok[3])
                perm = [int(v) for v in tok[5:]]
                assert len(perm) == W
                perms.append((seed, t, W, perm))
    return keys, perms
