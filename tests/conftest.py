import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def load_hand_cases(path):
    """Parse tests/golden/hand_cases.txt into a list of dicts."""
    import numpy as np
    cases, cur = [], None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            if key == "case":
                cur = {"name": vals[0], "m": int(vals[1]), "n": int(vals[2]), "d": int(vals[3])}
                cases.append(cur)
            elif key == "rows":
                cur["rows"] = np.array([float(v) for v in vals], np.float32).reshape(
                    cur["m"], cur["n"], cur["d"])
            elif key == "eps":
                cur["eps"] = np.array([int(v) for v in vals], np.int8).reshape(cur["m"], cur["n"] // 2)
            elif key == "r":
                cur["r"] = np.array([float(v) for v in vals], np.float64)
            elif key == "perm":
                cur["perm"] = np.array([int(v) for v in vals], np.int32).reshape(cur["m"], cur["n"])
    return cases


def load_reorder_cases(path):
    import numpy as np
    out = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            s, p, e = [x.strip() for x in line.split("|")]
            signs = np.array([int(v) for v in s.split()], np.int8)
            perm_in = None if p == "-" else np.array([int(v) for v in p.split()], np.int32)
            expect = np.array([int(v) for v in e.split()], np.int32)
            out.append((signs, perm_in, expect))
    return out


GOLDEN = os.path.join(ROOT, "tests", "golden")
