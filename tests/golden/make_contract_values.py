#!/usr/bin/env python3
"""Writes tests/golden/contract_values.txt: worked values of the operator contract, evaluated with
the arbitrary-precision Python rendering of the definitions in oracle/brute.py (and nothing else:
neither the C oracle nor the HIP library is involved).  Run from the repository root:

    python tests/golden/make_contract_values.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import brute  # noqa: E402

HEADER = """# Worked values of the operator contract, obtained by evaluating the written
# definitions with arbitrary-precision Python integers when the contract was
# drafted (independently of the C oracle).  They are consequences of this
# repository's readings, not numbers printed in the paper (it prints none).
# Format: <name> <hex value>; seeds and messages are named in the test that reads this.
"""


def values():
    K = brute.mix64(7)
    a, b = brute.hash_bytes(1, b"abc"), brute.hash_bytes(2, b"xy")
    rows = [("hash_seed0_empty", brute.hash_bytes(0, b"")),
            ("hash_seed1_abc", a),
            ("hash_seeddeadbeef_hello", brute.hash_bytes(0xdeadbeef, b"hello")),
            ("hash_seed2_xy", b),
            ("mix64_0", brute.mix64(0)),
            ("mix64_1", brute.mix64(1)),
            ("mix64_7", K),
            ("cross_K7_abc_xy", brute.cross(K, a, b)),
            ("cross_K7_xy_abc", brute.cross(K, b, a)),
            ("bucket_sign_K7_idx3", brute.mix64((K + 3) & (2 ** 64 - 1)))]
    for k, tok in enumerate(b"x,y,,z".split(b",")):
        rows.append((f"field1_seed11_tok{k}", brute.hash_bytes(11, tok)))
    return rows


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "contract_values.txt")
    with open(path, "w") as f:
        f.write(HEADER)
        for name, v in values():
            f.write(f"{name} {v:x}\n")
    print(path)
