"""Writes tests/golden/topdown_td64.json: what the CPU checker generates for the `td64` workload, per tree (number of
nodes, greatest depth, smallest |score| of any of its nodes).  Calls only the checker and the seeded input
generators; takes about a minute.  Run from the repository root:  python tests/golden/make_topdown_golden.py
"""
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
import oracle  # noqa: E402
from paper_1809_00832_amd import synth  # noqa: E402


def main():
    w = synth.topdown_workload("td64")
    r = oracle.td_generate(w.u_td, w.b_td, w.w_stop, w.b_stop, w.h_root, w.c_root, w.max_depth, w.max_nodes)
    n, B = r["n_nodes"], w.h_root.shape[0]
    tree = np.arange(n)
    for v in range(B, n):
        tree[v] = tree[r["parent"][v]]
    out = {"workload": "td64", "n_nodes": int(n), "truncated": int(r["truncated"]),
           "per_depth": [int(x) for x in np.bincount(r["depth"])],
           "trees": [{"nodes": int((tree == t).sum()), "depth": int(r["depth"][tree == t].max()),
                      "min_abs_score": float(np.abs(r["score"][tree == t]).min())} for t in range(B)]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "topdown_td64.json")
    with open(path, "w") as fh:
        json.dump(out, fh, indent=1)
    print("wrote", path, "nodes", n)


if __name__ == "__main__":
    main()
