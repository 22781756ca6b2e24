"""Reader for the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _ints(s):
    return [int(v) for v in s.split()]


def read_hand_examples():
    path = os.path.join(GOLDEN_DIR, "hand_example_def1_def2.txt")
    examples, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = {}
                examples[line.strip("[]")] = cur
                continue
            key, val = [p.strip() for p in line.split("=", 1)]
            if key in ("alpha", "beta"):
                cur[key] = float(val)
            elif key == "A":
                cur[key] = np.array([[float(v) for v in row.split()] for row in val.split(";")])
            elif key.startswith("token_sets"):
                cur[key] = [_ints(row) for row in val.split(";")]
            else:
                cur[key] = _ints(val)
    return examples
