"""Writes tests/golden/oracle_small.txt from the CPU oracle alone.

The paper prints no worked numerical example, so this fixture is not a pin of
the oracle against the paper (the closed forms and invariants in
tests/test_oracle_pins.py are); it freezes the oracle's output on one tiny
seeded case per variant so that a later change to the oracle's arithmetic
shows up as a diff.  Calls only oracle/ and the seeded input generator.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import attention  # noqa: E402
from paper_2502_15349_amd.workloads import BY_ID, make_inputs  # noqa: E402

CASES = {
    1: dict(L_q=5, L_k=5, D_qk=8, D_v=8, B=1, H_q=2, H_kv=2),
    2: dict(L_q=6, L_k=6, D_qk=8, D_v=8, B=1, H_q=4, H_kv=2),
    3: dict(L_q=6, L_k=6, D_qk=8, D_v=8, B=1, H_q=2, H_kv=2),
    4: dict(L_q=6, L_k=6, D_qk=8, D_v=16, B=1, H_q=2, H_kv=2),
    5: dict(L_q=4, L_k=7, D_qk=24, D_v=16, B=1, H_q=2, H_kv=2),
}


def compute(cid):
    w = BY_ID[cid].scaled(**CASES[cid])
    Q, K, V = make_inputs(w)
    O = attention(Q, K, V, scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                  gamma=w.gamma(), norm=w.norm, mask=w.mask)
    return w, O


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/ only; first row of head 0 per case\n")
        for cid in sorted(CASES):
            w, O = compute(cid)
            f.write(f"{cid} " + " ".join(f"{x:.15e}" for x in O[0, 0, -1]) + "\n")


if __name__ == "__main__":
    main()
