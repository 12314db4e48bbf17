"""Writes tests/golden/alpha_star.txt from the oracle alone (run from the repo root).

The paper defines alpha* (Sec. 3.1, "Gaussian Fitting") but prints no value, so the stored
table is the oracle's own derivation; the HIP library's built-in constants are tested
against it.  Columns: bits, alpha*, minimal Gaussian MSE, P(M = 0) on N(0,1).
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import alpha_star as a  # noqa: E402

with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "alpha_star.txt"), "w") as f:
    f.write("# bits alpha_star gaussian_mse untrusted_fraction  (oracle/alpha_star.py; Sec. 3.1, 3.2)\n")
    for bits in (1, 2, 3, 4, 8):
        alpha = a.alpha_star(bits)
        f.write(f"{bits} {alpha:.7f} {a.gaussian_mse(alpha, bits):.9e} "
                f"{a.untrusted_fraction(alpha, bits):.6e}\n")
    alpha = a.alpha_star_fp4()
    f.write("# FP4 grid (Sec. 4.4): alpha_star_fp4 gaussian_mse untrusted_fraction at T = alpha / 6\n")
    f.write(f"fp4 {alpha:.7f} {a.gaussian_mse_fp4(alpha):.9e} "
            f"{2.0 * float(a.ndtr(-alpha * (1.0 + a.FP4_TRUST))):.6e}\n")
