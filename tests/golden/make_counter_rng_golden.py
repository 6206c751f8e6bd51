"""Writes tests/golden/counter_rng_golden.txt: keys and uniforms of the oracle's counter-based generator at a few
(seed, purpose tag, sequence, position, index) points.  Imports only the oracle.  The file pins the bit pattern of
row_key / uniforms against later edits (a changed shift, constant or tag); the finaliser underneath is pinned to
the published splitmix64 stream separately (splitmix64_seed0.txt).

    python tests/golden/make_counter_rng_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import deer_oracle as O  # noqa: E402

POINTS = [  # (seed, tag, seq, pos, idx)
    (0, 1, 0, 0, 0), (0, 2, 0, 0, 0), (0, 3, 0, 0, 0), (4, 1, 0, 64, 151935), (4, 2, 15, 32768, 0),
    (4, 3, 15, 32799, 1023), (77, 1, 3, 4096, 7), ((1 << 64) - 1, 3, 1023, (1 << 31) - 1, (1 << 20) + 5),
    (123456789012345, 2, 255, 1 << 20, 99),
]


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "counter_rng_golden.txt")
    with open(path, "w") as f:
        f.write("# seed tag seq pos idx -> row_key (hex), uniforms(row_key, idx) * 2^23 - 0.5 (the 23 random bits, integer)\n")
        f.write("# written by tests/golden/make_counter_rng_golden.py from oracle/deer_oracle.py\n")
        for seed, tag, seq, pos, idx in POINTS:
            key = int(O.row_key(seed, tag, seq, pos))
            r = float(O.uniforms(key, idx)) * 8388608.0 - 0.5
            assert r == int(r)
            f.write(f"{seed} {tag} {seq} {pos} {idx} 0x{key:016X} {int(r)}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
