"""Writes tests/golden/mask_tiny_seed0.txt from the CPU oracle alone.

The file records this build's mask convention on the smallest workload
(4x4 blocks, seed 0, stream 0, p = 0.5): the sixteen 32-bit words that decide
the blocks, the keep flags and the packed 64-bit row words.  It is a
regression fixture for the convention, not a value from the paper (the paper
does not specify a generator; Section 3.4 only says the mask is sampled in
C++ and bit-packed).  Run:  python tests/golden/make_mask_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import sdrop_oracle as orc  # noqa: E402


def main():
    MB = KB = 4
    seed = stream = 0
    p = 0.5
    words = [orc.block_word(seed, stream, b) for b in range(MB * KB)]
    keep = orc.mask(MB, KB, p, seed, stream)
    packed = orc.pack_bits(keep)
    with open(os.path.join(HERE, "mask_tiny_seed0.txt"), "w") as f:
        f.write("# written by tests/golden/make_mask_golden.py from oracle/ only\n")
        f.write("# MB=4 KB=4 seed=0 stream=0 p=0.5 threshold=%d\n" % orc.threshold(p))
        f.write("words " + " ".join(str(w) for w in words) + "\n")
        f.write("keep " + " ".join(str(int(v)) for v in keep.reshape(-1)) + "\n")
        f.write("packed " + " ".join(hex(int(v)) for v in packed.reshape(-1)) + "\n")


if __name__ == "__main__":
    main()
