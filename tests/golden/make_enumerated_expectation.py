"""Writes tests/golden/enumerated_expectation.txt: the exact expected number of
activated experts E[N] for tiny (E, K, t), by enumerating every way t tokens can
each pick a K-subset of E experts (the uniform-routing model of Sec. 3.2) and
counting distinct experts.  Pure Python integers and fractions; calls nothing
from the oracle or the GPU library, so it pins both from outside."""
import itertools
import os
from fractions import Fraction

CASES = [(4, 1, 1), (4, 1, 3), (4, 2, 1), (4, 2, 2), (4, 2, 3), (5, 2, 3), (5, 3, 2),
         (6, 2, 3), (6, 3, 2), (6, 1, 4), (3, 3, 2), (8, 2, 2)]


def enumerate_expectation(E, K, t):
    subsets = list(itertools.combinations(range(E), K))
    total = 0
    n = 0
    for pick in itertools.product(subsets, repeat=t):
        active = set()
        for s in pick:
            active.update(s)
        total += len(active)
        n += 1
    return Fraction(total, n)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "enumerated_expectation.txt")
    with open(out, "w") as f:
        f.write("# E K t numerator denominator  (exact E[N], uniform K-subsets; Sec. 3.2 model)\n")
        for E, K, t in CASES:
            fr = enumerate_expectation(E, K, t)
            f.write(f"{E} {K} {t} {fr.numerator} {fr.denominator}\n")
    print(out)
