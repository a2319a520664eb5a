"""Writes tests/golden/generator_first8.txt: the first eight draws of each distribution for a few
(seed, tensor) pairs.  Calls only the input generator (no oracle, no GPU code).  Run from the repo
root:  python tests/golden/make_generator_golden.py
The file freezes the generator's definition so that a later edit cannot silently change every
workload's operands."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from paper_2605_28213_amd import inputs as gen  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "generator_first8.txt")

with open(OUT, "w") as f:
    f.write("# kind seed tensor : eight values as C99 hex floats (fp32 values, exact)\n")
    for seed in (0, 1, 2):
        for tensor in (gen.TENSOR_A, gen.TENSOR_B):
            u = gen.uniform_pm1(seed, tensor, 8)
            z = gen.normal(seed, tensor, 8, 1.0)
            f.write(f"uniform {seed} {tensor} : " + " ".join(float(v).hex() for v in u) + "\n")
            f.write(f"normal {seed} {tensor} : " + " ".join(float(v).hex() for v in z) + "\n")
print("wrote", OUT)
