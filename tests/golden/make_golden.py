#!/usr/bin/env python3
"""Writes oracle_traj_c1.txt from the CPU oracle alone (calls nothing but `oracle/` and the seeded
input generators).  The file freezes the oracle's arithmetic: a later change to it shows up as a
diff here and must be justified from the paper.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle       # noqa: E402
import workloads    # noqa: E402

COLS = [0, 1, 2, 3, 1000, 4095]   # columns of workload 1 that are stored


def trajectories():
    w = workloads.get("c1_ring4")
    topo = oracle.topology(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    x0 = workloads.x0(w)[:, COLS]
    grads = [workloads.grad(w, k)[:, COLS] for k in range(w.steps)]
    out = {}
    for algo in ("decentlam", "dmsgd"):
        x, m = oracle.run(algo, x0, lambda k, _x: grads[k], topo, gamma, beta, w.steps, storage="fp32")
        out[algo] = (x.astype(np.float32), m.astype(np.float32))
    return out


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_traj_c1.txt")
    with open(path, "w") as f:
        f.write("# Workload c1_ring4 (n=4, ring, gamma=0.1, beta=0.9), state after 10 iterations of the CPU oracle\n")
        f.write("# (Algorithm 1 and Algorithm 2 in fp64, fp32 storage between iterations), columns %s.\n" % COLS)
        f.write("# Written by tests/golden/make_golden.py from oracle/ only; values are C99 hex floats.\n")
        for algo, (x, m) in trajectories().items():
            for name, arr in (("x", x), ("m", m)):
                for i in range(arr.shape[0]):
                    f.write(f"{algo} {name} {i}: " + " ".join(float(v).hex() for v in arr[i]) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
