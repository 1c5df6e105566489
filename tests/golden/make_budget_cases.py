"""Writes tests/golden/budget_cases.txt from the oracle only (never from the HIP library)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import pkv_oracle  # noqa: E402

CASES = [  # (L, avg, beta, alpha)
    (4, 128, 20, 8), (32, 128, 20, 8), (32, 64, 20, 32), (32, 128, 20, 32), (32, 512, 20, 32),
    (32, 2048, 20, 32), (32, 256, 20, 16), (80, 128, 20, 64), (3, 100, 7, 5), (1, 77, 20, 8),
    (5, 40, 1, 8), (7, 8, 20, 8), (32, 96, 14, 8), (80, 2048, 16, 48),
]

with open(os.path.join(HERE, "budget_cases.txt"), "w") as f:
    f.write("# L avg beta alpha : k_0 .. k_{L-1}   (written by make_budget_cases.py from oracle/ only)\n")
    for (L, avg, beta, alpha) in CASES:
        k = pkv_oracle.budgets(L, avg, beta, alpha)
        f.write(f"{L} {avg} {beta} {alpha} : " + " ".join(str(int(x)) for x in k) + "\n")
