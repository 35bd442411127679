"""Writes the App. E Eq. "budget" values stored in paper_values.txt.

B/n = 1 - (1 - 2^-K)^L - L 2^-K (1 - 2^-K)^(L-1), evaluated exactly with rationals and
rounded once to a double.  Uses nothing but the standard library.
"""
from fractions import Fraction


def budget(K, L):
    x = Fraction(1, 2 ** K)
    return float(1 - (1 - x) ** L - L * x * (1 - x) ** (L - 1))


if __name__ == "__main__":
    for K, L in ((10, 150), (8, 75), (9, 120), (10, 170)):
        print(f"budget_K{K}_L{L} {budget(K, L)!r}")
