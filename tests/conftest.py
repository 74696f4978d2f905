import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden_mask(name):
    """Read tests/golden/<name>: '#' lines are comments, 'key = int' lines are the
    pattern parameters, the remaining lines are rows of 0/1 (row = query)."""
    import numpy as np
    params, rows = {}, []
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if "=" in line:
                k, v = line.split("=")
                params[k.strip()] = int(v)
            else:
                rows.append([int(c) for c in line])
    return params, np.array(rows, dtype=np.uint8)


GOLDEN_MASKS = ["mask_sink_window_token.txt", "mask_block_strided.txt", "mask_token_strided.txt"]
