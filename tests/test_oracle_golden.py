"""The oracle still produces the frozen bit patterns of tests/golden/oracle_step_golden.txt."""
import numpy as np

import oracle
from golden_util import load_cases


def test_oracle_reproduces_its_golden_file():
    cases = load_cases()
    assert len(cases) == 4
    for c in cases:
        p, m, v = c["in_p"].copy(), c["in_m"].copy(), c["in_v"].copy()
        lp = np.zeros(p.size, np.uint16)
        cfg = oracle.config(**c["kw"])
        sumsq, flag = (None, 0)
        if c["use_norm"]:
            sumsq, flag = oracle.grad_sumsq([c["in_g"]], c["dtype"])
            assert sumsq == c["sumsq"] and flag == 0
        oracle.adamw(p, m, v, c["in_g"], lp, c["dtype"], cfg, sumsq, flag)
        for got, key in ((p, "out_p"), (m, "out_m"), (v, "out_v")):
            assert np.array_equal(got.view(np.uint32), c[key].view(np.uint32)), (c["name"], key)
        assert np.array_equal(lp, c["out_lp"]), c["name"]
