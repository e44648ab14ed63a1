"""Writes tests/golden/hash_kat.txt: known-answer vectors of the random source.

Calls only the CPU oracle.  Run from the repository root:
    python tests/golden/make_hash_kat.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

CASES = [(0, 0, 0), (0, 0, 1), (0, 1, 0), (1, 0, 0), (1 << 32, 0, 0), (0xDEADBEEFCAFEF00D, 12345, 6789),
         (2 ** 64 - 1, 2 ** 31 - 1, 2 ** 31 - 1), (2, 970751, 6271), (0x0000000200000010, 77, 1567),
         (42, 3, 2 ** 24), (7, 2 ** 20, 2 ** 16 + 1), (0x123456789ABCDEF0, 1, 1),
         (3, 0, 0), (3, 65535, 1567), (4, 1, 2), (0x8000000000000000, 0x40000000, 0x40000000)]

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hash_kat.txt")
with open(out, "w") as fh:
    fh.write("# Known-answer vectors of the codec's counter-based random source (paper names no\n"
             "# generator; this build's definition).  seed plane pair_index -> 32-bit word.\n"
             "# Written by tests/golden/make_hash_kat.py from the CPU oracle; the test also\n"
             "# re-derives every line with an independent Python big-integer evaluation.\n")
    for c in CASES:
        fh.write("0x%016x %d %d 0x%08x\n" % (c[0], c[1], c[2], oracle.hash32(*c)))
print("wrote", out)
