"""Writes tests/golden/noise_bits.txt from the oracle alone (never the GPU path)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import kf_oracle as ko  # noqa: E402

TUPLES = []
for seed in (0, 1, 20240309, 0xDEADBEEFCAFEF00D, 2**64 - 1):
    for layer, head in ((0, 0), (1, 0), (0, 1), (27, 15), (31, 31)):
        for q_pos, k_pos in ((0, 0), (1, 0), (0, 1), (127, 64), (2048, 2047), (34815, 32767),
                             (2**31 - 1, 2**31 - 1)):
            TUPLES.append((seed, layer, head, q_pos, k_pos))

if __name__ == "__main__":
    with open(os.path.join(HERE, "noise_bits.txt"), "w") as f:
        f.write("# seed layer head q_pos k_pos bits  (all decimal)\n")
        for t in TUPLES:
            f.write("%d %d %d %d %d %d\n" % (*t, ko.noise_bits(*t)))
    print("wrote", len(TUPLES), "rows")
