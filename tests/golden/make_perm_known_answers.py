"""Writes tests/golden/perm_known_answers.txt from the CPU oracle alone (Section 3.2 permutation:
32-bit xorshift keys, sorted with the coordinate index as tie-break).  The file freezes the
constants of the key generator so that an accidental change to either side is caught."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

CASES = [(0, 0, 16), (1, 0, 1000), (180306333, 2, 4097), (2 ** 64 - 1, 7, 100000)]

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "perm_known_answers.txt")
with open(out, "w") as f:
    f.write("# kind seed chunk m first-16-values ; written by make_perm_known_answers.py from oracle/ only\n")
    for seed, chunk, m in CASES:
        perm, keys = oracle.permutation(seed, m, chunk=chunk, want_keys=True)
        f.write("keys %d %d %d %s\n" % (seed, chunk, m, " ".join(str(int(k)) for k in keys[:16])))
        f.write("perm %d %d %d %s\n" % (seed, chunk, m, " ".join(str(int(k)) for k in perm[:16])))
print(out)
