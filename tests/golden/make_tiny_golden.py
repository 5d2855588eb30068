"""Writes tests/golden/tiny_oracle.txt from the oracle alone (no GPU code).

Guards the oracle against silent drift: the file holds, for the Tiny workload
(1 layer, d 256, 4 heads x 64, FFN 688; one device, 64 prompt rows as 4 chunks
of 16, then verify segments of 4 rows at starts 64, 66, 70), each step's
output sum, sum of squares and three sampled elements, in float64.
Run from the repo root:  python tests/golden/make_tiny_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import hat_inputs as hi            # noqa: E402
from oracle import OracleMiddle    # noqa: E402

SEED = 1000


def tiny_outputs():
    cfg = hi.TINY
    m = OracleMiddle(cfg, [hi.layer_weights(cfg, 0, SEED)])
    outs = []
    for i, step in enumerate(hi.tiny_schedule()):
        dev, kind, start, n = step[0]
        x = hi.hidden_rows(n, cfg["d_model"], SEED, i)
        outs.append(m.forward([(dev, start, x)])[0])
    return outs


def rows(outs):
    for i, y in enumerate(outs):
        yield "%d %.15e %.15e %.15e %.15e %.15e" % (i, y.sum(), (y * y).sum(), y[0, 0], y[-1, 7], y[y.shape[0] // 2, 255])


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.txt")
    with open(path, "w") as f:
        f.write("# step sum sumsq y[0,0] y[-1,7] y[n/2,255]  (written by make_tiny_golden.py from oracle/ only)\n")
        f.write("\n".join(rows(tiny_outputs())) + "\n")
    print("wrote", path)
