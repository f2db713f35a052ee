"""Pure-Python fingerprint (oracle, test infrastructure; tiny inputs only).

Python integers are unbounded, so every step reduces modulo 2^64 explicitly.
This is the brute-force counterpart of ``oracle.c``: same definition, written
a second time in a language with different integer semantics, so that a
width, shift or overflow slip in either shows up as a disagreement.

The fingerprint indexes the Tensor Mapping (paper Section 3.1, which leaves
the function open; the function is the position-keyed SplitMix64 sum fixed by
the build's problem statement).
"""

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def splitmix64_py(x: int) -> int:
    """SplitMix64 output for a state ``x`` that has not been advanced yet."""
    z = (x + GAMMA) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def fingerprint_py(data: bytes, first_index: int = 0) -> int:
    """Wrapping sum of SM(w_i XOR i*gamma) over little-endian 8-byte words.

    Bytes past the end read as zero; the empty input gives 0.  ``first_index``
    numbers the first word (0 for a whole tensor); a non-zero value gives the
    partial sum of a slice that starts at that word of a longer tensor.
    """
    total = 0
    n = len(data)
    words = (n + 7) // 8
    for i in range(words):
        chunk = data[8 * i:8 * i + 8]
        w = int.from_bytes(chunk.ljust(8, b"\0"), "little")
        key = ((first_index + i) * GAMMA) & MASK64
        total = (total + splitmix64_py(w ^ key)) & MASK64
    return total
