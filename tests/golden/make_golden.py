"""Writes tests/golden/fingerprints.txt from the CPU oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
Every stored value comes from oracle.fingerprint (the C loop); nothing here
imports or calls the HIP library.  The inputs are described by a tiny recipe
language so the test can rebuild them:
    zeros:<nbytes>            nbytes zero bytes
    bf16one:<nbytes>          the bf16 constant 1.0 (0x3F80, little endian) repeated
    words:<a>,<b>,...         little-endian 64-bit words
    ramp:<nbytes>             byte j holds (j*131 + 7) mod 256
"""
import os
import struct
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402

RECIPES = [
    "zeros:0", "zeros:8", "zeros:16", "zeros:24", "zeros:4096",
    "bf16one:8", "bf16one:16", "bf16one:512", "bf16one:4096", "bf16one:8192",
    "bf16one:16384", "words:1,2", "words:2,1", "words:1", "ramp:1", "ramp:7",
    "ramp:9", "ramp:1000", "ramp:65537", "ramp:1048583",
]


def build(recipe: str) -> bytes:
    kind, arg = recipe.split(":")
    if kind == "zeros":
        return bytes(int(arg))
    if kind == "bf16one":
        return b"\x80\x3f" * (int(arg) // 2)
    if kind == "words":
        return b"".join(struct.pack("<Q", int(w)) for w in arg.split(","))
    if kind == "ramp":
        return bytes((j * 131 + 7) % 256 for j in range(int(arg)))
    raise ValueError(recipe)


def main() -> None:
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fingerprints.txt")
    with open(out, "w") as f:
        f.write("# recipe fingerprint(hex); written by make_golden.py from oracle.fingerprint\n")
        for r in RECIPES:
            f.write("%s 0x%016X\n" % (r, oracle.fingerprint(build(r))))


if __name__ == "__main__":
    main()
