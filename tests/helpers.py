"""Small helpers shared by the tests (no method arithmetic)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def random_fp16(rng, shape, kind="normal"):
    if kind == "normal":
        x = rng.standard_normal(shape)
    elif kind == "wide":
        x = rng.standard_normal(shape) * np.exp(rng.uniform(-8, 8, shape))
    elif kind == "positive":
        x = np.abs(rng.standard_normal(shape)) * 100 + 1000
    elif kind == "tiny":
        x = rng.standard_normal(shape) * 1e-6
    else:
        raise ValueError(kind)
    return np.clip(x, -60000, 60000).astype(np.float16)
