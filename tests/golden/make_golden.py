"""Writes tests/golden/pattern_table.txt from the oracle alone (a regression
lock on the pattern order; it calls nothing but oracle/).  Run from the repo
root:  python tests/golden/make_golden.py"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

here = os.path.dirname(os.path.abspath(__file__))
tab = oracle.pattern_table()
with open(os.path.join(here, "pattern_table.txt"), "w") as f:
    f.write("# id  uint16 encoding (bit 4i+j = m_ij) of the legal 4x4 blocks, in the order\n")
    f.write("# 'lexicographic on the row-major string m00..m33, 0 < 1'.  The count, 90, is the\n")
    f.write("# paper's n_t (Sec. 5.1, step 1).  Written by make_golden.py from oracle/ only.\n")
    for k, v in enumerate(tab):
        f.write(f"{k} 0x{int(v):04X}\n")
print("wrote", len(tab), "patterns")
