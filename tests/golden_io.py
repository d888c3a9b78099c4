"""Reader for the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_kv(name):
    """Lines 'key v v ; v v' -> dict key -> 2-D (or 1-D) float array, or a string."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, rest = line.split(None, 1)
            try:
                rows = [[float(v) for v in r.split()] for r in rest.split(";")]
            except ValueError:
                out[key] = rest.strip()
                continue
            out[key] = np.array(rows if len(rows) > 1 else rows[0], dtype=np.float64)
    return out
