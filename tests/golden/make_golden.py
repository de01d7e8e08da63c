"""Writes tests/golden/ihelm_f64_n3_E2.txt from the CPU oracle (and nothing else)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import numpy as np  # noqa: E402

import oracle  # noqa: E402
from paper_2604_19906_amd import workloads as wl  # noqa: E402


def main():
    w = wl.custom(3, 2, "f64", key=77)
    u, sx, sy, sz, d = wl.make_inputs(w)
    v = oracle.ihelm_apply(u, sx, sy, sz, d)
    path = os.path.join(HERE, "ihelm_f64_n3_E2.txt")
    with open(path, "w") as f:
        f.write("# oracle.ihelm_apply on workloads.custom(3, 2, 'f64', key=77); "
                "v[e,i,j,k] in C order, hex floats\n")
        for x in v.ravel():
            f.write(float(x).hex() + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
