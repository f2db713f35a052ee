"""Pins for the oracle's fingerprint (CPU only).

The fingerprint indexes the Tensor Mapping (paper Section 3.1).  Nothing in
this file retypes the mix: expected values come from published SplitMix64
vectors, from sums of those vectors, from an independent computation made
when the build was specified, from algebra (inverses computed with pow()),
and from the pure-Python brute force on tiny inputs.
"""
import os
import random
import struct

import pytest

import oracle
from oracle import fingerprint, fingerprint_py, splitmix64, splitmix64_py
from recipes import build, read_pairs

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = os.path.join(HERE, "golden")
M64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def published():
    vec = {}
    with open(os.path.join(GOLD, "splitmix64_vectors.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            seed, j, val = line.split()
            vec[(int(seed), int(j))] = int(val, 0)
    return vec


@pytest.mark.parametrize("impl", [splitmix64, splitmix64_py])
def test_mix_matches_published_vectors(impl):
    for (seed, j), val in published().items():
        assert impl((seed + j * GAMMA) & M64) == val


@pytest.mark.parametrize("impl", [fingerprint, fingerprint_py])
def test_zero_tensor_is_sum_of_generator_outputs(impl):
    # w_i = 0 makes term i equal to output i of the generator seeded with 0.
    vec = published()
    acc = 0
    assert impl(b"") == 0
    for w in range(3):
        acc = (acc + vec[(0, w)]) & M64
        assert impl(bytes(8 * (w + 1))) == acc


@pytest.mark.parametrize("impl", [fingerprint, fingerprint_py])
def test_xor_keying_and_word_order(impl):
    # Choose w_i so that w_i XOR i*gamma is the state that yields published
    # output i for seed 1234567: the sum must be the sum of those outputs.
    vec = published()
    words = [((i * GAMMA) & M64) ^ ((1234567 + i * GAMMA) & M64) for i in range(5)]
    want = sum(vec[(1234567, i)] for i in range(5)) & M64
    data = b"".join(struct.pack("<Q", w) for w in words)
    assert impl(data) == want
    # add-keying or a swapped word order would break this
    swapped = b"".join(struct.pack("<Q", w) for w in reversed(words))
    assert impl(swapped) != want
    # a constant state s in every position gives W * SM(s)
    for w in (1, 2, 7, 64):
        data = b"".join(struct.pack("<Q", ((i * GAMMA) & M64) ^ 1) for i in range(w))
        assert impl(data) == (w * vec[(1, 0)]) & M64


@pytest.mark.parametrize("impl", [fingerprint, fingerprint_py])
def test_little_endian_words_and_zero_padded_tail(impl):
    vec = published()
    assert impl(b"\x01" + bytes(7)) == vec[(1, 0)]
    assert impl(b"\x01") == vec[(1, 0)]            # missing bytes read as 0
    assert impl(bytes(7) + b"\x01") != vec[(1, 0)]
    rnd = random.Random(5)
    for n in range(1, 40):
        b = bytes(rnd.randrange(1, 256) for _ in range(n))
        pad = (-n) % 8
        assert impl(b) == impl(b + bytes(pad))
        if pad:
            assert impl(b) != impl(b + b"\x01" + bytes(pad - 1))
        # one more zero *word* changes the sum by SM(W * gamma): not neutral
        assert impl(b + bytes(pad)) != impl(b + bytes(pad + 8))


def test_values_computed_when_the_build_was_specified():
    for recipe, val in read_pairs(os.path.join(GOLD, "specified_fingerprints.txt")):
        assert fingerprint(build(recipe)) == val, recipe
        assert fingerprint_py(build(recipe)) == val, recipe


def test_stored_golden_file_is_current():
    for recipe, val in read_pairs(os.path.join(GOLD, "fingerprints.txt")):
        data = build(recipe)
        assert fingerprint(data) == val, recipe
        if len(data) <= 70000:
            assert fingerprint_py(data) == val, recipe


def test_c_loop_equals_pure_python_on_every_small_length():
    rnd = random.Random(1357)
    for n in list(range(0, 130)) + [255, 256, 257, 1023, 4099]:
        b = bytes(rnd.getrandbits(8) for _ in range(n))
        assert fingerprint(b) == fingerprint_py(b), n


def test_identical_bytes_identical_fingerprint_and_position_dependence():
    rnd = random.Random(2)
    b = bytes(rnd.getrandbits(8) for _ in range(4096))
    assert fingerprint(b) == fingerprint(bytes(bytearray(b)))
    w = [struct.pack("<Q", 1), struct.pack("<Q", 2)]
    assert fingerprint(w[0] + w[1]) != fingerprint(w[1] + w[0])


def test_every_single_bit_flip_changes_the_fingerprint():
    rnd = random.Random(3)
    for n in (1, 8, 13, 40):
        b = bytearray(rnd.getrandbits(8) for _ in range(n))
        base = fingerprint(bytes(b))
        seen = {base}
        for bit in range(8 * n):
            b[bit // 8] ^= 1 << (bit % 8)
            f = fingerprint(bytes(b))
            assert f != base
            seen.add(f)
            b[bit // 8] ^= 1 << (bit % 8)
        assert len(seen) == 8 * n + 1


def test_split_at_a_word_boundary_adds_up():
    # The property tiled reductions rely on: partial sums over word ranges,
    # each keyed with its absolute word index, add to the whole.
    rnd = random.Random(4)
    b = bytes(rnd.getrandbits(8) for _ in range(8 * 37 + 5))
    whole = fingerprint(b)
    for cut_words in (0, 1, 5, 36, 37):
        head = fingerprint_py(b[:8 * cut_words])
        tail = fingerprint_py(b[8 * cut_words:], first_index=cut_words)
        assert (head + tail) & M64 == whole
    # three-way split in arbitrary order of summation
    parts = [fingerprint_py(b[0:80]), fingerprint_py(b[80:160], 10),
             fingerprint_py(b[160:], 20)]
    assert sum(reversed(parts)) & M64 == whole


def _unxorshift(z, s):
    x = z
    for _ in range(64 // s + 1):
        x = z ^ (x >> s)
    return x


def invert_mix(y):
    """Inverse of the mix, from modular inverses and xor-shift inversion."""
    m1 = pow(0xBF58476D1CE4E5B9, -1, 1 << 64)
    m2 = pow(0x94D049BB133111EB, -1, 1 << 64)
    z = _unxorshift(y, 31)
    z = (z * m2) & M64
    z = _unxorshift(z, 27)
    z = (z * m1) & M64
    z = _unxorshift(z, 30)
    return (z - GAMMA) & M64


def colliding_pair(seed=11, words=4):
    """Two different byte strings of equal length with equal fingerprints."""
    rnd = random.Random(seed)
    terms = [rnd.getrandbits(64) for _ in range(words)]
    d = rnd.getrandbits(63) | 1
    other = list(terms)
    other[0] = (other[0] + d) & M64
    other[-1] = (other[-1] - d) & M64

    def to_bytes(ts):
        return b"".join(struct.pack("<Q", invert_mix(t) ^ ((i * GAMMA) & M64))
                        for i, t in enumerate(ts))
    return to_bytes(terms), to_bytes(other)


def test_mix_is_a_bijection_and_collisions_can_be_built():
    rnd = random.Random(6)
    for _ in range(200):
        x = rnd.getrandbits(64)
        assert invert_mix(splitmix64(x)) == x
    a, b = colliding_pair()
    assert a != b and len(a) == len(b)
    assert fingerprint(a) == fingerprint(b)
    assert not oracle.bytes_equal(a, b)


def test_bytes_equal_and_copy():
    import numpy as np
    rnd = random.Random(7)
    a = bytes(rnd.getrandbits(8) for _ in range(1000))
    assert oracle.bytes_equal(a, bytes(bytearray(a)))
    for pos in (0, 1, 500, 999):
        b = bytearray(a)
        b[pos] ^= 0x10
        assert not oracle.bytes_equal(a, bytes(b))
    assert not oracle.bytes_equal(a, a[:-1])
    dst = np.zeros(1000, dtype=np.uint8)
    oracle.copy_bytes(dst, a)
    assert dst.tobytes() == a
