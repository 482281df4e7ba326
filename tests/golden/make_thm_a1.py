"""Writes thm_a1_relative_error.txt: the closed form of Theorem A.1
(Appendix A.1), sqrt(p - 2 (t_p/sigma) phi(t_p/sigma)) with t_p the p-quantile
of |X| for X ~ N(0, sigma^2), evaluated at the sparsity levels the paper's
tables use.  Uses only the formula (no oracle, no GPU code)."""
import math
import os

from scipy.stats import norm

LEVELS = (0.25, 0.40, 0.50, 0.65, 0.80, 0.90)


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                       "thm_a1_relative_error.txt")
    with open(out, "w") as f:
        f.write("# Theorem A.1 (Appendix A.1): E||Y - Yhat|| / E||Y|| for independent\n"
                "# Gaussian X, W under magnitude sparsification at level p, sigma_X = 1.\n"
                "# columns: p  t_p = Phi^-1((1+p)/2)  sqrt(p - 2 t_p phi(t_p))\n")
        for p in LEVELS:
            t = norm.ppf((1.0 + p) / 2.0)
            f.write(f"{p:.2f} {t:.6f} {math.sqrt(p - 2.0 * t * norm.pdf(t)):.6f}\n")


if __name__ == "__main__":
    main()
