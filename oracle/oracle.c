/*
 * CPU oracle for the byte-level steps of the Load path (test infrastructure).
 *
 * This file is a checker, not part of the product: only tests, the smoke
 * check and the benchmark's cpu_baseline leg may build, load or call it.  It
 * shares no source, header, table or helper with the HIP library and is kept
 * deliberately plain: scalar loops in the order of the definition, no
 * blocking, no vectorisation hints, no threads.
 *
 * What it defines
 *  - tgo_splitmix64 / tgo_fingerprint: the content fingerprint that indexes
 *    the Tensor Mapping (the paper's Section 3.1 asks for one fingerprint per
 *    tensor and leaves the function open; the function used here is the
 *    position-keyed SplitMix64 sum fixed by the build's problem statement).
 *  - tgo_bytes_equal: bytewise identity, the reuse criterion behind the
 *    fingerprint (Section 3.1: a tensor found in the mapping is reused).
 *  - tgo_copy: the definition of assembling a tensor into its slot
 *    (Section 3.1: after loading, every tensor of the model is at its
 *    returned address).
 */
#include <stddef.h>
#include <stdint.h>

#define TGO_GAMMA 0x9E3779B97F4A7C15ULL

/* SplitMix64 output function applied to a state that has not yet been
 * advanced: advance by the golden-ratio increment, then two xor-shift /
 * multiply rounds and a final xor-shift.  All arithmetic is modulo 2^64. */
uint64_t tgo_splitmix64(uint64_t x)
{
    uint64_t z = x + TGO_GAMMA;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* F(b[0..n)) = sum over i in [0, ceil(n/8)) of SM(w_i XOR (i * gamma)),
 * where w_i is the little-endian 64-bit word made of bytes 8i .. 8i+7 and
 * bytes past the end of the tensor read as zero.  F of the empty tensor is 0.
 * The word is built byte by byte so the result does not depend on the
 * endianness or alignment rules of the machine running the oracle. */
uint64_t tgo_fingerprint(const uint8_t *b, uint64_t n)
{
    uint64_t words = n / 8 + (n % 8 != 0);
    uint64_t sum = 0;
    for (uint64_t i = 0; i < words; ++i) {
        uint64_t w = 0;
        for (unsigned j = 0; j < 8; ++j) {
            uint64_t at = 8 * i + j;
            uint64_t byte = at < n ? b[at] : 0;
            w |= byte << (8 * j);
        }
        sum += tgo_splitmix64(w ^ (i * TGO_GAMMA));
    }
    return sum;
}

/* 1 when the two extents hold the same n bytes, else 0. */
int tgo_bytes_equal(const uint8_t *a, const uint8_t *b, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i)
        if (a[i] != b[i])
            return 0;
    return 1;
}

/* dst[0..n) = src[0..n); the extents do not overlap. */
void tgo_copy(uint8_t *dst, const uint8_t *src, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i)
        dst[i] = src[i];
}
