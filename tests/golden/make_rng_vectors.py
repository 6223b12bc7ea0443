"""Writes tests/golden/rng_vectors.txt from the CPU oracle only.

The GPU library's host-side key derivation and draw function are checked
against this file (they are a second, independent implementation of the same
generator).  Run from the repository root: python tests/golden/make_rng_vectors.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle as orc  # noqa: E402

P61 = (1 << 61) - 1
HERE = os.path.dirname(os.path.abspath(__file__))

lines = ["# key seed domain stream_id party j -> key ; draw key e -> 64-bit output, field element mod 2^61-1"]
cases = [(0, 1, 0, 0, 1), (1, 1, 0, 0, 1), (1, 2, 0, 3, 2), (0xDEADBEEF, 3, 151, 0, 2),
         (2 ** 64 - 1, 7, 2 ** 40, 5, 1), (12345, 4, 9, 0, 0), (12345, 5, 9, 0, 1), (12345, 6, 9, 0, 2)]
for c in cases:
    k = orc.key(*c)
    lines.append("key " + " ".join(str(v) for v in c) + f" {k}")
    for e in (0, 1, 2 ** 28 - 1, 2 ** 40 + 17):
        lines.append(f"draw {k} {e} {orc.draw(k, e)} {orc.draw_field(k, e, P61)}")
open(os.path.join(HERE, "rng_vectors.txt"), "w").write("\n".join(lines) + "\n")
print(len(lines), "lines")
