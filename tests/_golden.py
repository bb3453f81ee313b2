"""Reader for tests/golden/adamw_hand_worked.txt ("[case]" headers, "key: values")."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

_VEC = ("grad", "master", "exp_avg", "exp_avg_sq")


def load_hand_worked():
    cases, cur = {}, None
    with open(os.path.join(GOLDEN, "adamw_hand_worked.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = cases.setdefault(line.strip("[]"), {})
                continue
            key, val = line.split(":", 1)
            toks = val.split()
            if key in _VEC or key.startswith("expect_") and len(toks) > 1:
                cur[key] = np.array([float(t) for t in toks], dtype=np.float64)
            elif key == "dtype":
                cur[key] = toks[0]
            else:
                cur[key] = float(toks[0])
    return cases
