"""Helpers shared by the tests (fixture parsing, error norms)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    """Parse 'key v v v' / 'device i: v v' lines into a dict of lists of floats/ints."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("device"):
                head, vals = line.split(":")
                out.setdefault("device", {})[int(head.split()[1])] = [int(v) for v in vals.split()]
            else:
                k, *vals = line.split()
                out[k] = [float(v) if ("." in v or "e" in v) else int(v) for v in vals]
    return out


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))
