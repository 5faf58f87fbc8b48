"""Writes tests/golden/noise_words.txt from the CPU oracle alone (never from the GPU path).

The noise function is this project's own definition (the paper's synthetic tensors are
noiseless, Sec. 5.1), so there is no published value to cite; the file freezes the
definition so that an accidental edit of the oracle's generator is caught.
Run:  python tests/golden/make_noise_golden.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

CASES = [(0x231113693000, 0, 0, 0), (0x231113693000, 1, 0, 0), (0x231113693000, 2, 0, 0),
         (0x231113693000, 3, 0, 0), (0x231113693000, 4, 0, 0), (0x231113693000, 0, 1, 0),
         (0x231113693000, 0, 0, 1), (0x231113693004, 9999, 9999, 9999), (1, 12345, 678, 9),
         (0xFFFFFFFFFFFFFFFF, 7, 7, 7), (0x100000000, 6, 5, 4)]

if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "noise_words.txt")
    with open(out, "w") as f:
        f.write("# seed i j k hash_word(hex) g(seed;i,j,k) -- written by make_noise_golden.py from oracle/ only\n")
        for seed, i, j, k in CASES:
            f.write("%#x %d %d %d %08x %.17g\n" % (seed, i, j, k, oracle.noise_word(seed, i, j, k),
                                                  oracle.noise(seed, i, j, k)))
    print(out)
