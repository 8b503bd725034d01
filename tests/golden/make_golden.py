"""Writes tests/golden/config1_fit.txt from the CPU oracle alone (never from the HIP path).

The file pins the oracle against accidental changes of its arithmetic: final centers, cluster
sizes and the fp64 objective after each of the 5 iterations of configuration 1 (Alg. 1).
Run:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads as W  # noqa: E402


def compute():
    w = W.CONFIGS[1]
    codes = W.codes_numpy(w)
    cent = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(W.codewords(w))
    lines = []
    for it in range(w.iters):
        a, _ = oracle.assign(codes, cent, tables)
        obj = oracle.objective(codes, cent, a, tables)
        cent, _, counts = oracle.update(codes, a, tables, cent)
        lines.append(f"iter {it} objective {obj:.6f} empty {int((counts == 0).sum())}")
    lines.append("centers " + cent.tobytes().hex())
    lines.append("counts " + " ".join(map(str, counts.tolist())))
    return lines


if __name__ == "__main__":
    with open(os.path.join(HERE, "config1_fit.txt"), "w") as f:
        f.write("# written by tests/golden/make_golden.py from the CPU oracle (configuration 1, Alg. 1, 5 iterations)\n")
        f.write("\n".join(compute()) + "\n")
