"""Writes tests/golden/synth_vectors.txt: the first 8 bf16 draws (std 0.02) of tensor stream 0 for the
three model seeds.  Calls only the input generator."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from paper_2603_20661_amd import synth  # noqa: E402

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "synth_vectors.txt")
with open(out, "w") as f:
    f.write("# seed stream  first 8 bf16 bit patterns of normal_bf16(seed, stream, std=0.02); written by make_synth_vectors.py\n")
    for seed in (0, 1, 2):
        v = synth.normal_bf16(seed, 0, 8, std=0.02)
        f.write(f"{seed} 0 " + " ".join(f"{x:04x}" for x in v) + "\n")
