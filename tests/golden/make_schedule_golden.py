"""Writes tests/golden/schedule_rank_lists.txt from the schedule oracle (and nothing else):
one line per (P, W, M, rank) with the rank's ordered task list, for the five BASELINE
configurations (every rank) and a few small cases.  Run from the repository root:
    python tests/golden/make_schedule_golden.py
"""

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import schedule as S  # noqa: E402

CASES = [(2, 1, 4), (4, 2, 8), (4, 1, 16), (16, 2, 32), (8, 4, 64), (3, 2, 5), (1, 2, 3), (5, 3, 2), (4, 2, 3)]


def main():
    out = os.path.join(ROOT, "tests", "golden", "schedule_rank_lists.txt")
    with open(out, "w") as f:
        f.write("# P W M rank : K<mb>.<chunk> ...   (written by make_schedule_golden.py from oracle/schedule.py)\n")
        for (P, W, M) in CASES:
            sim = S.simulate(P, W, M)
            for r in range(P):
                toks = " ".join("%s%d.%d" % ("FB"[t.kind], t.mb, t.chunk) for t in sim["lists"][r])
                f.write("%d %d %d %d : %s\n" % (P, W, M, r, toks))
    print("wrote", out)


if __name__ == "__main__":
    main()
