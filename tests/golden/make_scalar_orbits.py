"""Writes tests/golden/scalar_orbits.txt: orbits of the scalar quintic.

On a matrix with singular values sigma_i, one Newton-Schulz iteration (Eq. 2,
section 2.1) maps every sigma_i to f(sigma_i) = a s + b s^3 + c s^5 and leaves the
singular vectors alone.  The orbit f^k(sigma) for k = 1..5 is computed here in
exact rational arithmetic (fractions.Fraction) from the coefficients the paper
states, (a, b, c) = (3.4445, -4.7750, 2.0315), and printed to 15 decimals.

Runs on the CPU with the standard library only; it calls neither the oracle nor
the HIP library.   Usage:  python tests/golden/make_scalar_orbits.py
"""
from fractions import Fraction
from pathlib import Path

A = Fraction(34445, 10000)
B = Fraction(-47750, 10000)
C = Fraction(20315, 10000)
STARTS = ["1", "4/5", "3/5", "1/2", "1/10", "1/100", "1/1000", "1/4", "9/10"]


def f(x: Fraction) -> Fraction:
    return A * x + B * x ** 3 + C * x ** 5


def dec(x: Fraction, digits: int = 15) -> str:
    scaled = round(x * 10 ** digits)
    sign = "-" if scaled < 0 else ""
    scaled = abs(scaled)
    return f"{sign}{scaled // 10 ** digits}.{scaled % 10 ** digits:0{digits}d}"


def main() -> None:
    lines = ["# sigma0  f(sigma0)  f^2  f^3  f^4  f^5   (Eq. 2 on singular values; coefficients of section 2.1)"]
    for s in STARTS:
        x = Fraction(s)
        row = [s]
        for _ in range(5):
            x = f(x)
            # keep the exact value but cap the denominator growth: 40 digits is far below 1e-15
            x = x.limit_denominator(10 ** 40)
            row.append(dec(x))
        lines.append("  ".join(row))
    Path(__file__).with_name("scalar_orbits.txt").write_text("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
