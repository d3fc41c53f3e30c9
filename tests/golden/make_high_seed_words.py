"""Writes the reference words for 64-bit seeds whose HIGH word is not zero (the seed-key step
K0 = mix32(lo ^ C1), K1 = mix32(hi ^ K0 ^ C2) of this repository's reading of "a seed", paper
Section 5.2) in the format of spec_words.txt.  It calls only the oracle.

    python tests/golden/make_high_seed_words.py            # prints the lines

The lines committed in spec_words.txt were also obtained, before being added there, from a
separate throw-away transcription of the written steps (plain Python integers, no oracle code);
the two agreed.  A slip in how the oracle (or the library) uses the high word changes K1 and
fails test_spec_words_fixture.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import blockperm as O  # noqa: E402

SEEDS = (1 << 32, 0xDEADBEEF12345678, 0xFFFFFFFFFFFFFFFF)

if __name__ == "__main__":
    for seed in SEEDS:
        k0, k1 = O.seed_keys(seed)
        print(f"keys {seed} = 0x{k0:08X} 0x{k1:08X}")
    for seed in SEEDS:
        a, b = O.wiring(1024, O.seed_keys(seed)[1])
        print(f"wiring {seed} 1024 = {a} {b}")
