#!/usr/bin/env python3
"""Writes tests/golden/attn_jvp_tiny.json: a tiny seeded attention + JVP problem and the fp64 oracle's answer.

The paper prints no worked example for App. C.1 / Alg. 2, so this fixture is not a pin of the oracle (its pins are
the closed forms, library routines and finite differences in tests/test_oracle_pins.py); it freezes the oracle's
output so that a later change to its arithmetic shows up as a diff of this file.  Calls only `oracle/`.
Run from the repository root:  python tests/golden/make_attn_jvp_tiny.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle.attn_jvp_ref import attn_jvp_ref_head      # noqa: E402
from oracle.rmsnorm_jvp_ref import rmsnorm_jvp_ref     # noqa: E402


def main():
    g = np.random.default_rng(20251008)
    Lq, Lkv, d, scale = 3, 5, 4, 0.5
    # values with short binary expansions (multiples of 1/8), so the text file holds them exactly
    draw = lambda *shape: np.round(g.normal(size=shape) * 8) / 8
    q, k, v, tq, tk, tv = draw(Lq, d), draw(Lkv, d), draw(Lkv, d), draw(Lq, d), draw(Lkv, d), draw(Lkv, d)
    o, to, lse = attn_jvp_ref_head(q, k, v, tq, tk, tv, scale)
    w, eps = draw(d) + 1.0, 0.125
    y, ty = rmsnorm_jvp_ref(q, tq, w, eps)
    out = {"scale": scale, "eps": eps,
           "inputs": {n: x.tolist() for n, x in dict(q=q, k=k, v=v, tq=tq, tk=tk, tv=tv, w=w).items()},
           "attention": {"o": o.tolist(), "to": to.tolist(), "lse": lse.tolist()},
           "rmsnorm_of_q": {"y": y.tolist(), "ty": ty.tolist()}}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_jvp_tiny.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
