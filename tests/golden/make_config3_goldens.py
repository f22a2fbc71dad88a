#!/usr/bin/env python3
"""Writes the stored expected values for the back-end loops at config-3 size, from the CPU oracle alone.

  config3_dstar.json   D* and the path recovery table that Algorithm "Remove Switch Nodes" (Appendix E.2) leaves on
                       config 3 (DGX-A100-shaped, 128 compute nodes, 17 switches) scaled to its optimum: capacities
                       U * b_e with U = 15, k = 2 trees per compute node (1/x* = 15/2, Proposition 3)
  config3_trees.json   the out-trees that Algorithm "Spanning Tree Construction" (Appendix E.3) builds on that D*

Both follow the visiting order the oracle documents (switches, egress heads, ingress tails in increasing id order;
root-sets in creation order, the first edge in (x, y) order with mu > 0), which makes the result unique, so the HIP
library's output can be compared element by element.  Imports `oracle` and `workloads` only; takes a few minutes
(about 4 million max-flows on one core).  Run from the repository root:  python tests/golden/make_config3_goldens.py
"""
import json
import os
import sys
from fractions import Fraction

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np          # noqa: E402

import oracle as o          # noqa: E402
import workloads as w       # noqa: E402

U, K = 15, 2


def main():
    t3 = w.config_topology(3)
    inv = o.optimality_binary_search(t3, threads=8)
    Uq, kq = o.smallest_U_k(inv, t3.bandwidth)          # (15/2, 1): on integers, capacities 15 * b_e and k = 2
    assert inv == Fraction(15, 2) and Uq * 2 == U and kq * 2 == K
    D = w.Topology(t3.name, t3.n_vertices, t3.tail, t3.head,
                   (np.asarray(t3.bandwidth, dtype=np.int64) * U).astype(np.int32), t3.is_compute)
    Dstar, table = o.remove_switches(D, K)
    links = o.link_capacities(Dstar)
    dstar = {"source": "oracle.remove_switches on workloads.config_topology(3) with capacities 15 * b_e, k = 2",
             "U": U, "k": K,
             "links": [[int(a), int(b), int(c)] for (a, b), c in sorted(links.items())],
             "table": [[int(u), int(t), int(sw), int(amount)] for (u, t), row in sorted(table.items()) for sw, amount in sorted(row.items())]}
    with open(os.path.join(HERE, "config3_dstar.json"), "w") as f:
        json.dump(dstar, f, separators=(",", ":"))
        f.write("\n")
    comp = [int(v) for v in t3.compute_nodes]
    idx = {v: i for i, v in enumerate(comp)}
    star = {(idx[a], idx[b]): c for (a, b), c in links.items()}
    trees = o.construct_trees(len(comp), star, K)
    out = {"source": "oracle.construct_trees on the D* of config3_dstar.json (compute nodes renumbered 0..127 in id order), k = 2",
           "n": len(comp), "k": K,
           "trees": [[int(root), int(mult), [int(v) for e in edges for v in e]] for root, mult, edges in trees]}
    with open(os.path.join(HERE, "config3_trees.json"), "w") as f:
        json.dump(out, f, separators=(",", ":"))
        f.write("\n")
    print(f"D*: {len(dstar['links'])} links, {len(dstar['table'])} table rows; {len(out['trees'])} root-sets")


if __name__ == "__main__":
    main()
