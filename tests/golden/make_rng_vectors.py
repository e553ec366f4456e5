"""Writes tests/golden/rng_vectors.txt: values of the synthetic-randomness
generator, evaluated from its written specification with Python integers
(arbitrary precision, reduced mod 2^64 by hand).  It calls neither the C oracle
nor the GPU library, so both can be held against the file.

Specification (not from the paper; the paper's randomness comes from its
OT-based offline phase, Section 4.2):
    mix(z):  z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;
             z *= 0x94D049BB133111EB; z ^= z>>31            (all mod 2^64)
    absorb(h, v)  = mix(h + (v+1)*0x9E3779B97F4A7C15)
    rand64(seed, stream, party, idx)
                  = absorb(absorb(absorb(absorb(0, seed), stream), party), idx)

Usage: python tests/golden/make_rng_vectors.py
"""
import os

M64 = (1 << 64) - 1


def mix(z):
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & M64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & M64
    z ^= z >> 31
    return z


def absorb(h, v):
    return mix((h + (v + 1) * 0x9E3779B97F4A7C15) & M64)


def rand64(seed, stream, party, idx):
    return absorb(absorb(absorb(absorb(0, seed), stream), party), idx)


CASES = [(0, 0, 0, 0), (0, 0, 0, 1), (1, 2, 3, 4), (0x5350494E01, 1, 1, 0),
         (0x5350494E05, 5, 4, (1 << 24) - 1), (M64, M64, 7, M64), (42, 8, 2, 1 << 40),
         (0x5350494E02, 6, 0, 12345), (0x5350494E02, 7, 1, 12345), (0x5350494E02, 8, 1, 12345)]

if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "rng_vectors.txt")
    with open(path, "w") as fh:
        fh.write("# seed stream party idx rand64   (hex; written by make_rng_vectors.py)\n")
        for c in CASES:
            fh.write("%x %x %x %x %016x\n" % (c + (rand64(*c),)))
    print("wrote", path)
