"""Writes tests/golden/key_chain_vectors.txt from the CPU oracle alone (regression vectors for
the build's own choice of how seed, epoch and start index are folded into a 64-bit key; the
paper only says the dataset is shuffled at the start of each epoch, Sec. 4.2)."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

lines = [
    "# Regression vectors written by make_key_vectors.py from the CPU oracle (not from the paper:",
    "# Sec. 4.2 fixes no generator).  key <seed> <epoch> <i> <hex key> | perm <seed> <epoch> <n> <order>",
]
for seed, epoch in [(0, 0), (7, 0), (7, 2)]:
    for i in range(3):
        lines.append(f"key {seed} {epoch} {i} {oracle.key(seed, epoch, i):016x}")
for seed, epoch, n in [(0, 0, 8), (7, 0, 8), (7, 1, 8)]:
    lines.append(f"perm {seed} {epoch} {n} " + ",".join(map(str, oracle.epoch_perm(seed, epoch, n).tolist())))
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "key_chain_vectors.txt"), "w") as fh:
    fh.write("\n".join(lines) + "\n")
