"""Writes tests/golden/zipf_bias_skewed.txt: the router's second bias for the skewed-load
workload (expert popularity ~ Zipf(1.2) over 32 experts), calibrated with the fp64 oracle
router on the first 65 536 slices of that workload.  Calls only the input generator and
oracle/.  Run from the repository root:  python tests/golden/make_zipf_bias.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.zipf_bias import calibrate_zipf_bias, zipf_shares  # noqa: E402
from paper_2510_04286_amd import workload as wl  # noqa: E402


def main():
    cfg = wl.CONFIGS["skewed"]
    w = wl.make_weights(cfg)
    n_slices = 65536
    h = wl.make_h(cfg, t0=0, t1=n_slices // cfg.S)
    x = h.reshape(-1, cfg.ds)
    bias, shares, it, err = calibrate_zipf_bias(x, w["Wr1"], w["br1"], w["Wr2"], cfg.k, cfg.zipf_s,
                                                wl.round_to_bf16)
    q = zipf_shares(cfg.E, cfg.zipf_s)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "zipf_bias_skewed.txt")
    with open(out, "w") as f:
        f.write("# router second-layer bias br2[32] (bf16-representable) for the skewed-load workload\n")
        f.write("# written by tests/golden/make_zipf_bias.py from the fp64 oracle router; target top-2\n")
        f.write(f"# selection shares Zipf(1.2); calibrated on {n_slices} slices, {it} iterations, "
                f"max |share/target - 1| = {err:.4f}\n")
        for e in range(cfg.E):
            f.write(f"{float(bias[e]):.9e}  # expert {e}: share {shares[e]:.5f} target {q[e]:.5f}\n")
    print("wrote", out, "iterations", it, "max rel err", err)


if __name__ == "__main__":
    main()
