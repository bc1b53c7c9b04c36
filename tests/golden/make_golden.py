"""Writes tests/golden/segment_small.json from the fp64 oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
The stored values are a regression guard for the oracle (Eq. 2 of Section 3 on a
fixed small case); they come from ``oracle/`` and from nothing else.  The paper
prints no worked numeric example, so there is no paper value to store.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2311_02382_amd import synth  # noqa: E402

CASE = dict(B=1, l_x=12, H=2, d=4, seed=77, s0=5, l_s=4, causal=True)


def main():
    c = CASE
    q, k, v, do = (a.astype(np.float64) for a in synth.make_inputs(c["B"], c["l_x"], c["H"], c["d"], c["seed"]))
    sl = slice(c["s0"], c["s0"] + c["l_s"])
    out, lse = oracle.segment_fwd(q[:, sl], k, v, c["s0"], c["causal"])
    dq, dk, dv = oracle.segment_bwd(q[:, sl], k, v, do[:, sl], c["s0"], c["causal"])
    doc = {"case": c, "cite": "Section 3, Principle 3, Eq. 2 (forward); textbook gradient (backward)",
           "out": out.ravel().tolist(), "lse": lse.ravel().tolist(), "dq": dq.ravel().tolist(),
           "dk_partial": dk.ravel().tolist(), "dv_partial": dv.ravel().tolist()}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "segment_small.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=0)
    print("wrote", path)


if __name__ == "__main__":
    main()
