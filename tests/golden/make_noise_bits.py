"""Write tests/golden/noise_bits.txt: worked values of the sampling-mode noise generator.

The generator is the one spelled out in include/aj.h under aj_verify_sampled (the paper's Appendix A,
"Generalization to sampling", asks only for Gumbel noise from a generator seeded by the random state
and the context, and names none).  The values here are worked out from that text with Python's
unbounded integers and exact fractions, every reduction mod 2^32 written out - no call into the CPU
oracle, none into the HIP library - so that the oracle's C implementation (and, through the parity
tests, the kernels') is tied to the published bit pattern and not only to its statistics.

usage: python tests/golden/make_noise_bits.py
"""
import os
from fractions import Fraction

HERE = os.path.dirname(os.path.abspath(__file__))
M32 = 1 << 32

CASES = [
    (0x0000000000000000, 0),
    (0x0000000000000000, 1),
    (0x0000000000000001, 0),
    (0x0000000100000000, 0),
    (0xFFFFFFFFFFFFFFFF, 128255),
    (0x0123456789ABCDEF, 40653),
    (0x8000000000000000, 77),
    (0x00000000FFFFFFFF, 16777215),
    (0xDEADBEEFCAFEF00D, 65536),
    (0x7FFFFFFFFFFFFFFF, 128000),
    (0x9E3779B97F4A7C15, 2),
    (0x000000000000002A, 16777221),     # v beyond 24 bits: the multiply is a full 32-bit one
]


def noise_bits(key: int, v: int) -> int:
    lo, hi = key % M32, key // M32
    h = (v * 0x9E3779 + lo) % M32
    h = h ^ (h // (1 << 16))
    h = (h * 0x85EBCA6B) % M32
    h = h ^ hi
    h = h ^ (h // (1 << 13))
    h = (h * 0xC2B2AE35) % M32
    h = h ^ (h // (1 << 16))
    h = (h * 0x27D4EB2F) % M32
    h = h ^ (h // (1 << 15))
    return h


def main():
    with open(os.path.join(HERE, "noise_bits.txt"), "w") as f:
        f.write("# sampling-mode noise generator (include/aj.h, aj_verify_sampled; Appendix A names no generator):\n")
        f.write("# worked with unbounded integers and exact fractions by tests/golden/make_noise_bits.py\n")
        f.write("# key(hex) v h(hex) n=h>>9 u=(n+1/2)/2^23 as numerator/2^24\n")
        for key, v in CASES:
            h = noise_bits(key, v)
            n = h >> 9
            u = Fraction(2 * n + 1, 1 << 24)
            assert 0 < u < 1 and u.denominator == 1 << 24
            f.write(f"{key:016x} {v} {h:08x} {n} {u.numerator}\n")


if __name__ == "__main__":
    main()
