"""Writes lemma1_counts.txt: Lemma 1's closed-form depth and product bound for n = s^k.

Pure arithmetic on the lemma's two formulas; calls nothing from the GPU path (and nothing
from the oracle either).  Run:  python tests/golden/make_lemma1_counts.py
"""
import os

rows = ["# Paper, Lemma 1: depth = 2k - 1, products <= ceil(2n / (s(s-1))) + 2k - 2  for n = s^k.",
        "# columns: s k n depth bound"]
for s, k in [(2, 4), (4, 1), (4, 2), (4, 3), (4, 5), (4, 6), (4, 14), (16, 1), (16, 2), (16, 3), (16, 4), (16, 6), (16, 7),
             (32, 1), (32, 2), (32, 3), (32, 5)]:
    n = s ** k
    bound = -(-2 * n // (s * (s - 1))) + 2 * k - 2
    rows.append(f"{s} {k} {n} {2 * k - 1} {bound}")
with open(os.path.join(os.path.dirname(__file__), "lemma1_counts.txt"), "w") as f:
    f.write("\n".join(rows) + "\n")
