"""Writes tests/golden/draw_values.txt: draws of the sampling generator for a few
(call seed, hop, node, slot) keys, computed by the CPU oracle alone.  The test that reads the
file recomputes every value with Python integers."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

KEYS = [
    (0, 0, 0, 0), (0, 0, 0, 1), (0, 1, 0, 0), (0, 0, 1, 0),
    (1234567, 0, 0, 0), (1234567, 1, 0, 0), (1234567, 0, 5, 0), (1234567, 0, 0, 5),
    (1234567, 2, 2449999, 14), (20211208, 1, 110999999, 9), (2**64 - 1, 7, 2**31 - 1, 63),
    (0x9E3779B97F4A7C15, 3, 42, 24), (2**63, 0, 2**30, 4), (987654321987654321, 5, 77, 31),
]

with open(os.path.join(HERE, "draw_values.txt"), "w") as f:
    f.write("# Draws of the counter-based sampling generator (reading: SplitMix64 steps keyed on call seed,\n"
            "# hop, node, slot), written by make_draw_golden.py from the CPU oracle.\n"
            "# call_seed hop node slot draw\n")
    for key in KEYS:
        f.write("%d %d %d %d %d\n" % (*key, oracle.draw(*key)))
print("wrote", len(KEYS), "values")
