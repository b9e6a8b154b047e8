#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ from the CPU oracle
(and from nothing else): a frozen record of what the oracle computes on a few
tiny seeded problems, so that a later change to its arithmetic shows up as a
diff of these files and has to be justified.  The values are NOT an independent
pin of the oracle (tests/test_oracle_pins.py holds those).

    python tests/golden/make_golden.py            # rewrite the fixtures
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import hyperattn_oracle as orc  # noqa: E402

CASES = {
    "unmasked_n32_d4": dict(n=32, d=4, b=8, m=6, r=3, causal=False, n_min=8, seed=7),
    "causal_n32_d4": dict(n=32, d=4, b=4, m=3, r=3, causal=True, n_min=8, seed=7),
}


def inputs(n, d):
    """Deterministic inputs without a random generator: smooth, irrational-looking values."""
    i = np.arange(n)[:, None].astype(np.float64)
    c = np.arange(d)[None, :].astype(np.float64)
    Q = np.sin(0.37 * i + 1.3 * c) * 0.9
    K = np.cos(0.23 * i - 0.7 * c) * 0.8
    V = np.sin(0.11 * i * (c + 1.0)) + 0.1 * c
    G = np.cos(0.19 * i + 0.5 * c)
    return (x[None, None] for x in (Q, K, V, G))


def compute(case):
    p = dict(CASES[case])
    n, d = p.pop("n"), p.pop("d")
    Q, K, V, G = inputs(n, d)
    out, lse = orc.hyperattn_forward(Q, K, V, **p)
    dQ, dK, dV = orc.hyperattn_backward(Q, K, V, G, **p)
    return {"out": out[0, 0], "lse": lse[0, 0], "dQ": dQ[0, 0], "dK": dK[0, 0], "dV": dV[0, 0],
            "R": orc.make_projection(p["seed"], d, p["r"]),
            "samples_level0": orc.make_samples(p["seed"], 0, 0, n // 2 if p["causal"] else n, p["m"])}


def main():
    for case in CASES:
        vals = compute(case)
        path = os.path.join(HERE, f"oracle_{case}.json")
        with open(path, "w") as f:
            json.dump({k: np.asarray(v).tolist() for k, v in vals.items()}, f, indent=0)
            f.write("\n")
        print("wrote", path)


if __name__ == "__main__":
    main()
