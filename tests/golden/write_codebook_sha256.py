"""Writes tests/golden/codebook_sha256.txt from the CPU oracle alone."""
import hashlib
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

HEADER = """# Regression fixture, NOT values printed by the paper: sha256 of the 1024-byte
# little-endian float32 table of each type, as produced by the closed forms of
# Sec. 3.1 (dynamic tree, linear, static tree, mantissa).  Written by
# tests/golden/write_codebook_sha256.py, which calls only oracle/.
"""

if __name__ == "__main__":
    with open(os.path.join(HERE, "codebook_sha256.txt"), "w") as f:
        f.write(HEADER)
        for kind in (0, 1, 2, 3):
            f.write("%d %s\n" % (kind, hashlib.sha256(oracle.codebook(kind).astype("<f4").tobytes()).hexdigest()))
