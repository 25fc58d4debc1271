import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU box)")


def read_plan_cases():
    """Parse tests/golden/chunk_plans.txt -> list of ((T, HW, chunk, overlap), rows)."""
    path = os.path.join(ROOT, "tests", "golden", "chunk_plans.txt")
    cases, cur = [], None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("case"):
                cur = (tuple(int(x) for x in line.split()[1:]), [])
                cases.append(cur)
            else:
                cur[1].append([int(x) for x in line.split()])
    return cases


@pytest.fixture(scope="session")
def plan_cases():
    return read_plan_cases()
