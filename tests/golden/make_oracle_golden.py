#!/usr/bin/env python3
"""Writes tests/golden/oracle_step_golden.txt: inputs and outputs of the CPU oracle, as bit patterns.

Calls nothing but oracle/ (and numpy for the seeded inputs).  The file freezes the oracle's behaviour: a
later change to its arithmetic shows up as a diff of this file and must be justified from the paper or
the standard definitions.  Run from the repository root:  python tests/golden/make_oracle_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_step_golden.txt")

CASES = [
    ("bf16_step1_adamw", oracle.BF16, dict(step=1), False),
    ("bf16_step10_adamw_clip", oracle.BF16, dict(step=10, max_grad_norm=0.01), True),
    ("fp16_step10_scale65536_clip", oracle.FP16, dict(step=10, loss_scale=65536.0, max_grad_norm=0.01), True),
    ("bf16_step100_adam_l2", oracle.BF16, dict(step=100, mode=oracle.MODE_ADAM_L2), False),
]


def inputs(name, dt, n=48):
    rng = np.random.default_rng(sum(map(ord, name)))
    p = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-4, n).astype(np.float32)
    v = np.abs(rng.normal(0, 1e-6, n)).astype(np.float32)
    gf = rng.normal(0, 1e-3, n).astype(np.float32)
    if "scale65536" in name:
        gf = gf * np.float32(65536.0)
    if "step1_" in name:
        m[:] = 0
        v[:] = 0
    # a few awkward elements
    gf[0] = 0.0
    m[1] = 0.0
    v[2] = 0.0
    p[3] = 0.0
    m[4] = np.float32(-(0.1 / 0.9)) * gf[4] / (np.float32(65536.0) if "scale65536" in name else np.float32(1))
    p[5] = np.float32(3e-5)
    v[6] = np.float32(1e-42)
    g = oracle.cast(gf, dt)
    return p, m, v, g


def main():
    lines = ["# Oracle golden values.  Written by tests/golden/make_oracle_golden.py (calls only oracle/).",
             "# case <name> dtype <0=bf16,1=fp16> then one line per array: hex bit patterns."]
    for name, dt, kw, use_norm in CASES:
        p, m, v, g = inputs(name, dt)
        cfg = oracle.config(**kw)
        sumsq, flag = oracle.grad_sumsq([g], dt) if use_norm else (None, 0)
        po, mo, vo = p.copy(), m.copy(), v.copy()
        lp = np.zeros(p.size, np.uint16)
        oracle.adamw(po, mo, vo, g, lp, dt, cfg, sumsq, flag)
        lines.append(f"case {name} dtype {dt} " + " ".join(f"{k}={val!r}" for k, val in sorted(kw.items()))
                     + f" use_norm={int(use_norm)}")
        if use_norm:
            lines.append("sumsq " + np.float64(sumsq).tobytes().hex())
        for label, arr in (("p", p), ("m", m), ("v", v)):
            lines.append(f"in_{label} " + " ".join(f"{x:08x}" for x in arr.view(np.uint32)))
        lines.append("in_g " + " ".join(f"{x:04x}" for x in g))
        for label, arr in (("p", po), ("m", mo), ("v", vo)):
            lines.append(f"out_{label} " + " ".join(f"{x:08x}" for x in arr.view(np.uint32)))
        lines.append("out_lp " + " ".join(f"{x:04x}" for x in lp))
    with open(OUT, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
