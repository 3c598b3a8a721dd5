"""Writes tests/golden/hash_words.txt from the CPU oracle alone (never from the HIP path).
Run:  python tests/golden/make_golden.py"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import ff_oracle as O  # noqa: E402

CASES = [(0, 0, 0), (0, 0, 1), (1, 0, 0), (0, 1, 0), (2, 5, 12345), (2, 5, (1 << 32) + 12345),
         (0xDEADBEEF, 1 << 20, 33554431), (7, (3 << 20) | (2 << 4) | (1 << 2) | 1, 999983)]

with open(os.path.join(HERE, "hash_words.txt"), "w") as f:
    f.write("# seed tag idx hash -- stochastic-rounding generator words, written by make_golden.py\n")
    f.write("# from oracle/ff_oracle.c (the paper fixes no generator: Section IV-B cites stochastic rounding only)\n")
    for s, t, i in CASES:
        f.write(f"{s:#x} {t:#x} {i:#x} {O.hash_u32(s, t, i):#010x}\n")
