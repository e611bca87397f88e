"""Writes tests/golden/tiny_oracle.json: what the float64 oracle computes for image 0 of the tiny
configuration.  The paper prints no worked numeric example, so this fixture is a regression anchor
written by the oracle alone (never by the HIP path):  python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import tokencarve_oracle as orc  # noqa: E402
from workloads import CONFIGS, make_image  # noqa: E402


def main():
    w = CONFIGS["tiny"]
    im = make_image(w, 0)
    out = orc.compress(im["Q"], im["K"], im["V"], im["X"][w.n_sys:w.n_sys + w.n_vis], w.n_sys, w.n_vis,
                       w.k_prune, w.k_final, lam=w.lam, dtype=w.dtype)
    doc = {
        "source": "oracle/tokencarve_oracle.py compress() on workloads tiny, image 0 (seed 10000)",
        "sigma": [float("%.12g" % v) for v in out["sigma"][:12]],
        "C": [float("%.12g" % v) for v in out["C"]],
        "S": [float("%.12g" % v) for v in out["S"]],
        "E": [float("%.12g" % v) for v in out["E"]],
        "order": [int(v) for v in out["order"]],
        "kept_idx": [int(v) for v in out["kept_idx"]],
        "merge_dst": [int(v) for v in out["merge_dst"]],
        "X_out_row0_first8": [float("%.9g" % v) for v in out["X_out"][0][:8]],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
