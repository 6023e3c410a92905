"""Writes tests/golden/alignment_counts.txt using only the brute-force enumerator in oracle/.

Each line: T  A  blank  label(comma separated, '-' if empty)  count
where count is the number of length-T strings over A symbols that the CTC operator
(Section 3.3, Eq. (ctc): Align(x, y)) maps to the label.  Run from the repo root:
    python tests/golden/make_golden.py
"""
import itertools
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import brute_force as bf  # noqa: E402


def main():
    rows = []
    for A, blank in ((2, 0), (3, 0), (3, 2), (4, 1)):
        nonblank = [k for k in range(A) if k != blank]
        for T in range(0, 7 if A < 4 else 6):
            for L in range(0, T + 2):
                for label in itertools.product(nonblank, repeat=L):
                    if L > 2 and hash(label) % 3:      # thin out, deterministic for ints
                        continue
                    rows.append((T, A, blank, label, bf.count_alignments(T, label, A, blank)))
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "alignment_counts.txt")
    with open(out, "w") as f:
        f.write("# T A blank label count -- enumerated by oracle/brute_force.py (CTC operator, Section 3.3 Eq. (ctc))\n")
        for T, A, blank, label, n in rows:
            f.write(f"{T} {A} {blank} {','.join(map(str, label)) or '-'} {n}\n")
    print(len(rows), "rows ->", out)


if __name__ == "__main__":
    main()
