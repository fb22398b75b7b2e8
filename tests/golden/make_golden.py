"""Writes the closed-form fixtures in this folder.

Nothing here calls the GPU library.  Values come from closed forms evaluated
with 50-digit arithmetic (mpmath) or from exact rational arithmetic.
Run:  python tests/golden/make_golden.py
"""
import os
from fractions import Fraction

import mpmath as mp

HERE = os.path.dirname(os.path.abspath(__file__))
mp.mp.dps = 50


def kms_logdet(n, rho):
    # det of the AR(1) / Kac-Murdock-Szego matrix rho^|i-j| is (1-rho^2)^(n-1)
    return (n - 1) * mp.log(1 - mp.mpf(rho) ** 2)


def hilbert_logdet(n):
    # exact determinant of the Hilbert matrix H_ij = 1/(i+j-1) by rational elimination
    a = [[Fraction(1, i + j + 1) for j in range(n)] for i in range(n)]
    det = Fraction(1)
    for k in range(n):
        det *= a[k][k]
        for i in range(k + 1, n):
            f = a[i][k] / a[k][k]
            for j in range(k, n):
                a[i][j] -= f * a[k][j]
    return mp.log(mp.mpf(det.numerator) / mp.mpf(det.denominator))


def main():
    with open(os.path.join(HERE, "kms_closed_form.txt"), "w") as fh:
        fh.write("# log det of the KMS / AR(1) matrix A_ij = rho^|i-j| :  (n-1) log(1-rho^2)\n")
        fh.write("# (textbook closed form; pivots of its LDL^T are 1, 1-rho^2, ..., 1-rho^2 and l_ij = rho^(i-j))\n")
        fh.write("# key = n_rho, value = logdet to 30 digits; written by make_golden.py with mpmath, 50 digits\n")
        for n, rho in ((512, "0.5"), (8192, "0.5"), (32768, "0.9"), (131072, "0.9"), (196608, "0.9"), (7, "0.3")):
            fh.write(f"{n}_{rho} {mp.nstr(kms_logdet(n, rho), 30)}\n")
    with open(os.path.join(HERE, "hilbert_logdet.txt"), "w") as fh:
        fh.write("# log det of the Hilbert matrix H_ij = 1/(i+j-1), exact rational elimination, 30 digits\n")
        for n in (3, 5, 8, 10):
            fh.write(f"{n} {mp.nstr(hilbert_logdet(n), 30)}\n")


if __name__ == "__main__":
    main()
