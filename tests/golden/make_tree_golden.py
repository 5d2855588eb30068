"""Writes tests/golden/tree_oracle.txt from the oracle alone (no GPU code).

Drift guard for the tree-verification path of the oracle: Tiny shapes (1 layer, d 256,
4 heads x 64, FFN 688), a 40-row prompt, then a tree of 8 candidates (the fixed shape
hat_inputs.MEDUSA_LIKE_TREE), the path to node 6 kept, and a chain of 3 after it.  The file
holds each step's output sum, sum of squares and three sampled elements, in float64.
Run from the repo root:  python tests/golden/make_tree_golden.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import hat_inputs as hi            # noqa: E402
from oracle import OracleMiddle    # noqa: E402

SEED = 1100


def tree_outputs():
    cfg = hi.TINY
    m = OracleMiddle(cfg, [hi.layer_weights(cfg, 0, SEED)])
    parents = hi.MEDUSA_LIKE_TREE
    path = hi.tree_path(parents, 6)
    outs = [m.forward([(0, 0, hi.hidden_rows(40, cfg["d_model"], SEED, 0))])[0],
            m.forward([(0, 40, hi.hidden_rows(8, cfg["d_model"], SEED, 1), hi.tree_masks(parents))])[0]]
    m.compact(0, 40, path)
    outs.append(m.forward([(0, 40 + len(path), hi.hidden_rows(3, cfg["d_model"], SEED, 2))])[0])
    return outs


def rows(outs):
    for i, y in enumerate(outs):
        yield "%d %.15e %.15e %.15e %.15e %.15e" % (i, y.sum(), (y * y).sum(), y[0, 0], y[-1, 7], y[y.shape[0] // 2, 255])


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tree_oracle.txt")
    with open(path, "w") as f:
        f.write("# step sum sumsq y[0,0] y[-1,7] y[n/2,255]  (written by make_tree_golden.py from oracle/ only)\n")
        f.write("\n".join(rows(tree_outputs())) + "\n")
    print("wrote", path)
