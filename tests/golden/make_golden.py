"""Writes tests/golden/tiny_layer.txt from the CPU oracle alone (no HIP code is
imported or run).  The paper prints no worked example of the MoE layer, so this
fixture is not a citation: it freezes the oracle's output on a hand-checkable
4-token layer so that an accidental change to the oracle's arithmetic shows up.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def tiny_inputs():
    # small exact binary fractions, so every printed digit is meaningful
    T, H, E, k, I = 4, 4, 4, 2, 2
    x = (np.arange(T * H).reshape(T, H) % 5 - 2).astype(np.float32) / 4
    gw = ((np.arange(E * H).reshape(E, H) * 3) % 7 - 3).astype(np.float32) / 4
    wg = ((np.arange(E * I * H).reshape(E, I, H) * 5) % 9 - 4).astype(np.float32) / 8
    wu = ((np.arange(E * I * H).reshape(E, I, H) * 7) % 11 - 5).astype(np.float32) / 8
    wd = ((np.arange(E * H * I).reshape(E, H, I) * 3) % 5 - 2).astype(np.float32) / 4
    return x, gw, {"w_gate": wg, "w_up": wu, "w_down": wd}, k


def compute():
    x, gw, W, k = tiny_inputs()
    ids, w, margin = oracle.route(x, gw, k)
    out, parts = oracle.layer_share(x, ids, w, 0, gw.shape[0], W)
    return ids, w, parts["offsets"], parts["perm"], out


if __name__ == "__main__":
    ids, w, offsets, perm, out = compute()
    with open(os.path.join(HERE, "tiny_layer.txt"), "w") as f:
        f.write("# oracle output on the 4-token layer of make_golden.py (not from the paper)\n")
        f.write("ids " + " ".join(map(str, ids.ravel())) + "\n")
        f.write("offsets " + " ".join(map(str, offsets)) + "\n")
        f.write("perm " + " ".join(map(str, perm)) + "\n")
        f.write("w " + " ".join("%.9g" % v for v in w.ravel()) + "\n")
        f.write("out " + " ".join("%.9g" % v for v in out.ravel()) + "\n")
