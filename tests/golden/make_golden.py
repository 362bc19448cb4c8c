"""Writes the stored expected values under tests/golden/.  Calls only oracle/.

worked_example_onehot.txt: the 3x3 ramp image 1..9, a single filter that is
one-hot at tap (0,0), R = 4 exact quarter turns, pad 1, all-ones upstream
gradient.  Rows 0-2 pooled output (Eq. 10), rows 3-5 argmax orientation,
rows 6-8 base-weight gradient (Eq. 14, 16), rows 9-11 input gradient (Eq. 13, 15).
The paper prints no numeric example; these follow from its equations and are
also asserted literally in tests/test_oracle_pins.py.
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import rotconv_oracle as orc  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    w = np.zeros((1, 1, 1, 3, 3))
    w[0, 0, 0, 0, 0] = 1.0
    _, yp, idx, _ = orc.layer_fwd(x, w, 4, pad=1)
    dx, dw = orc.layer_bwd(x, w, np.ones((1, 1, 3, 3)), idx, 4, pad=1)
    rows = np.concatenate([yp[0, 0], idx[0, 0].astype(np.float64), dw[0, 0, 0], dx[0, 0]], axis=0)
    np.savetxt(os.path.join(HERE, "worked_example_onehot.txt"), rows, fmt="%.1f",
               header="ramp 3x3, one-hot tap (0,0), R=4, pad 1: ypool(3) idx(3) dW(3) dX(3); Eq. 7,10,12-16")


if __name__ == "__main__":
    main()
