"""Writes tests/golden/schedule_vectors.txt from the CPU oracle only.

Usage: python tests/golden/make_schedule_vectors.py
Each line: pattern seed k L straggler_p  order[L] partner[L] active[L]."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import schedule as S  # noqa: E402

CASES = [(S.FIXED_RING, 0, 4, 0.0), (S.FIXED_RING, 5, 7, 0.25), (S.RANDOM_RING, 0, 8, 0.0),
         (S.RANDOM_RING, 0, 64, 0.1), (S.RANDOM_RING, 2**63 + 11, 16, 0.1), (S.D1D, 0, 16, 0.0)]

with open(os.path.join(HERE, "schedule_vectors.txt"), "w") as fh:
    fh.write("# written by make_schedule_vectors.py from oracle/schedule.py; the paper fixes no sequence\n")
    for pattern, seed, L, p in CASES:
        for k in (0, 1, 2, 49, 1000003):
            order, partner, active = S.schedule(pattern, seed, k, L, p)
            fh.write(" ".join(map(str, [pattern, seed, k, L, p] + order + partner + active)) + "\n")
