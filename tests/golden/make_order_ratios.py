"""Writes tests/golden/order_ratios.txt: for seeded traffic matrices on at most four GPUs, the
Theorem 2 / Theorem 4 bound, the smallest completion time over EVERY combination of per-GPU
whole-flow orders (brute force, the method the paper itself uses to judge its heuristic in
Sec. 8.2), and what Algorithm 1's order and the chosen send order reach.  Calls only the oracle.

    python tests/golden/make_order_ratios.py
"""
import os
import sys

from fractions import Fraction

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import schedule as S  # noqa: E402

RATES = (Fraction(1), Fraction(4, 5), Fraction(1, 2), Fraction(2, 5))   # the four link speeds of Sec. 8.1 over the fastest


def cases():
    r = np.random.default_rng(20241017)
    for n in (3, 3, 3, 3, 4, 4, 4, 4, 4, 4, 4, 4):
        for hetero in (False, True):
            D = r.integers(0, 12, size=(n, n))
            D[r.random((n, n)) < 0.25] = 0
            np.fill_diagonal(D, 0)
            B = [RATES[k] for k in r.integers(0, 4, size=n)] if hetero else None
            if S.bmax(D.tolist(), B) > 0:
                yield D.tolist(), B


def main():
    out = ["# D (rows separated by /) | B (- = all 1) | b_max | brute-force best | simulate(alg1 order) | send_order time",
           "# exact rationals; written by tests/golden/make_order_ratios.py from the oracle alone",
           "# b_max: Theorem 2 (Sec. 4.2) and, with unequal rates, Theorem 4 / Appendix B (Sec. 5.2); the orders: Algorithm 1",
           "# (Sec. 4.2) and the send order chosen among whole-flow candidates; best: exhaustion over all ((n-1)!)^n orders",
           "# under the fluid big-switch model of Sec. 3"]
    for D, B in cases():
        best, _ = S.brute_force_best_order(D, B)
        a = S.simulate(D, B, S.alg1_order(D, B)["dest_order"])
        s = S.send_order(D, B)["time"]
        out.append(" | ".join([" / ".join(" ".join(str(v) for v in row) for row in D),
                               "-" if B is None else " ".join(str(b) for b in B),
                               str(S.bmax(D, B)), str(best), str(a), str(s)]))
        print(out[-1], flush=True)
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "order_ratios.txt"), "w") as f:
        f.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
