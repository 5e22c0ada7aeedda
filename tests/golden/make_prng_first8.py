"""Writes tests/golden/prng_first8.txt: the first 8 draws of each distribution of the seeded input
generator (seed 260329011, tensor 1), as exact hexadecimal float64.  Calls the input generator only."""
import os
import sys

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from paper_2603_29010_amd import synth  # noqa: E402

SEED, TENSOR = synth.BASE_SEED + 1, 1


def rows():
    yield "uniform01", synth.uniform01(SEED, TENSOR, 8)
    yield "uniform_pm1", synth.uniform_pm1(SEED, TENSOR, 8)
    yield "normal", synth.normal(SEED, TENSOR, 8)
    yield "randint_m2_2", synth.randint(SEED, TENSOR, 8, -2, 2)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "prng_first8.txt")
    with open(out, "w") as f:
        f.write("# first 8 draws per distribution, seed 260329011, tensor 1 (float64, C99 hex); written by make_prng_first8.py\n")
        for name, v in rows():
            f.write(name + " " + " ".join(float(x).hex() for x in v) + "\n")
    print(out)
