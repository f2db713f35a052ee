"""Rebuilds the byte strings named by the recipes in tests/golden/*.txt."""
import struct


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


def read_pairs(path):
    out = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            out.append((parts[0], int(parts[1], 0)))
    return out
