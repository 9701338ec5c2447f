"""Reader of tests/golden/oracle_step_golden.txt (written by tests/golden/make_oracle_golden.py)."""
import os

import numpy as np

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_step_golden.txt")


def _val(s):
    try:
        return int(s)
    except ValueError:
        return float(s)


def load_cases():
    cases, cur = [], None
    for line in open(PATH):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, _, rest = line.partition(" ")
        if head == "case":
            tok = rest.split()
            cur = dict(name=tok[0], dtype=int(tok[2]), sumsq=None,
                       kw={k: _val(v) for k, v in (t.split("=") for t in tok[3:])})
            cur["use_norm"] = bool(cur["kw"].pop("use_norm"))
            cases.append(cur)
        elif head == "sumsq":
            cur["sumsq"] = float(np.frombuffer(bytes.fromhex(rest), np.float64)[0])
        else:
            words = rest.split()
            if head.endswith("_g") or head.endswith("_lp"):
                cur[head] = np.array([int(x, 16) for x in words], np.uint16)
            else:
                cur[head] = np.array([int(x, 16) for x in words], np.uint32).view(np.float32)
    return cases
