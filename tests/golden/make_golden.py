"""Writes tests/golden/lbscan_small_golden.json from the CPU oracle alone.

The paper prints no worked numerical example of the scan, so this fixture is not
a value from the paper: it freezes the oracle's output on one small seeded input,
so that an accidental change to the oracle's arithmetic shows up as a diff.
Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402


def small_problem():
    r = np.random.default_rng(424242)
    B, D, N, L = 1, 2, 3, 7
    return dict(
        x=r.standard_normal((B, D, L)), delta=0.5 * r.standard_normal((B, D, L)),
        A=-r.uniform(0.5, 2.0, size=(D, N)), Bm=r.standard_normal((B, N, L)),
        Cm=r.standard_normal((B, N, L)), Dskip=r.standard_normal(D),
        z=r.standard_normal((B, D, L)), delta_bias=r.uniform(-1.0, 0.0, size=D))


def main():
    p = small_problem()
    dout = np.random.default_rng(424243).standard_normal(p["x"].shape)
    out = {"window": 3, "fwd": oracle.fwd(**p, window=3).tolist(),
           "bidir_self": oracle.bidir_fwd(dict(p), dict(p)).tolist()}
    g = oracle.bwd(**p, dout=dout, window=3)
    out["bwd"] = {k: v.tolist() for k, v in g.items()}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lbscan_small_golden.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
