import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


GOLDEN = os.path.join(ROOT, "tests", "golden")


def read_hand_examples(path=os.path.join(GOLDEN, "eq123_hand_examples.txt")):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "case":
            cur = {"name": vals[0]}
        elif key == "end":
            cases.append(cur)
            cur = None
        elif key in ("alpha", "beta", "gamma", "tol"):
            cur[key] = float(vals[0])
        else:
            cur[key] = [float(v) for v in vals]
    return cases
