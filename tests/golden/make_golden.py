"""Writes the stored expected values under tests/golden/ from the CPU oracle (and nothing else)."""
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

    cw = wl.conv_custom(3, 2, "f64", key=78, nq=4)
    p, m, d_vq, i_vq = wl.conv_inputs(cw)
    f_ref = oracle.convection_apply(p, m, d_vq, i_vq)
    path = os.path.join(HERE, "convection_f64_nv3_nq4_E2.txt")
    with open(path, "w") as f:
        f.write("# oracle.convection_apply on workloads.conv_custom(3, 2, 'f64', key=78, nq=4); "
                "F[c,e,k,j,i] in C order, hex floats\n")
        for x in f_ref.ravel():
            f.write(float(x).hex() + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
