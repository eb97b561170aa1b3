"""Writes tests/golden/mix_golden.txt: the oracle's routing hash on fixed inputs (regression guard).

Calls only oracle/.  Run from the repository root:  python tests/golden/make_mix_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import np_oracle  # noqa: E402

KEYS = [0x0, 0x1, 0x2, 0x5FF, 0x600, 0xFFFFFFFF, 0x100000000, 0x2FAF07FF, 0x123456789ABCDEF,
        0x7FFFFFFFFFFFFFFF, 0x8000000000000000, 0xFFFFFFFFFFFFFFFF]

with open(os.path.join(HERE, "mix_golden.txt"), "w") as f:
    f.write("# key(hex) mix(key)(hex); the routing hash is a convention of this build, not a value from the paper\n")
    for k in KEYS:
        f.write(f"{k:016x} {np_oracle.mix(k):016x}\n")
