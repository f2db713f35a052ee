// Device kernels of the Load path for gfx950 (CDNA4, wave64).
//
// Three streaming kernels share one work decomposition.  A launch covers a
// table of extents (spans to fingerprint, pairs to compare, copies to make).
// Every extent is cut into tiles of TILE = 256 lanes x 16 bytes x U bytes;
// tiles of all extents are numbered consecutively and dealt round-robin to a
// fixed number of resident workgroups (tile t goes to workgroup t mod grid).
// Neighbouring workgroups therefore touch neighbouring 4U KiB pieces of HBM at
// any moment, which keeps all channels busy, and each lane issues U
// independent 128-bit loads before it consumes any of them.
//
// None of this is a dense contraction, so there is no MFMA here; nothing is
// reused across tiles, so the only data kept in LDS is the per-wave partial
// sum of the fingerprint's cross-wave combine.  The XCD a workgroup lands on
// does not matter for correctness or reuse (each tile is read once); the
// descriptor tables are a few KiB and end up in every XCD's L2.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tgk {

typedef unsigned long long u64;
typedef unsigned int u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;               // 4 waves of 64
constexpr u64 kGamma = 0x9E3779B97F4A7C15ull;

struct Span { u64 ptr, nbytes; };           // extent to fingerprint
struct Pair { u64 a, b, nbytes; };          // extents to compare
struct Copy { u64 dst, src, nbytes; };      // extent to copy (non-overlapping)

template <int U> constexpr u64 tile_bytes() { return u64(kThreads) * 16 * U; }

// SplitMix64 output function on a state that has not been advanced.
__device__ __forceinline__ u64 mix(u64 x) {
    u64 z = x + kGamma;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ u64 lohi(u32 lo, u32 hi) { return (u64(hi) << 32) | lo; }

// v + (v seen through a DPP lane permutation), for a 64-bit value held as two
// 32-bit halves.  CTRL is a DPP control word: 0x00-0xFF quad_perm, 0x141
// row_half_mirror, 0x140 row_mirror.
template <int CTRL> __device__ __forceinline__ u64 dpp_add(u64 v) {
    const int lo = __builtin_amdgcn_update_dpp(0, int(u32(v)), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, int(u32(v >> 32)), CTRL, 0xF, 0xF, false);
    return v + lohi(u32(lo), u32(hi));
}

// Sum of v over the 64 lanes of a wave; the result is wave-uniform.
// Butterfly inside each row of 16 lanes with DPP (lane^1, lane^2, mirror in 8,
// mirror in 16), then the four row sums are read out and added on the scalar
// unit.  Integer addition wraps and commutes, so any order is bit-exact.
__device__ __forceinline__ u64 wave_sum(u64 v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror: lane i <-> 7-i within 8
    v = dpp_add<0x140>(v);   // row_mirror: lane i <-> 15-i within 16
    u64 s = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const u32 lo = __builtin_amdgcn_readlane(int(u32(v)), row * 16);
        const u32 hi = __builtin_amdgcn_readlane(int(u32(v >> 32)), row * 16);
        s += lohi(lo, hi);
    }
    return s;
}

// Finds the extent that holds tile t.  prefix[s] is the number of tiles before
// extent s; prefix[n] the total.  Extents with zero tiles are skipped.
__device__ __forceinline__ u32 locate_first(const u32 *__restrict__ prefix, u32 n, u32 t) {
    u32 lo = 0, hi = n;       // invariant: prefix[lo] <= t < prefix[hi]
    while (hi - lo > 1) {
        const u32 mid = (lo + hi) >> 1;
        if (prefix[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ u32x4 load16(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
__device__ __forceinline__ void store16(void *p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

// Little-endian word made of up to 8 bytes at p; bytes at or past `avail` are 0.
__device__ __forceinline__ u64 tail_word(const uint8_t *p, u32 avail) {
    u64 w = 0;
    for (u32 j = 0; j < 8 && j < avail; ++j) w |= u64(p[j]) << (8 * j);
    return w;
}

// ---------------------------------------------------------------- fingerprint
// out[s] += sum over the words of span s of mix(w_i ^ i*gamma).  `out` must be
// zero before the launch.  Per-lane sums are carried across consecutive tiles
// of one span and folded (wave DPP reduce, LDS across the four waves, one
// 64-bit atomic per workgroup) only when the workgroup moves to another span.
template <int U>
__global__ __launch_bounds__(kThreads) void fingerprint_kernel(const Span *__restrict__ spans,
                                                                const u32 *__restrict__ prefix,
                                                                u32 n_spans, u64 *__restrict__ out) {
    constexpr u64 TILE = tile_bytes<U>();
    __shared__ u64 wave_part[kThreads / 64];
    const u32 total = prefix[n_spans];
    const u32 tid = threadIdx.x;
    u32 t = blockIdx.x;
    if (t >= total) return;

    u32 s = locate_first(prefix, n_spans, t);
    u32 first = prefix[s], next = prefix[s + 1];
    Span sp = spans[s];
    u64 acc = 0;

    auto fold = [&](u32 span_index) {
        const u64 w = wave_sum(acc);
        if ((tid & 63) == 0) wave_part[tid >> 6] = w;
        __syncthreads();
        if (tid == 0) {
            u64 sum = 0;
#pragma unroll
            for (int i = 0; i < kThreads / 64; ++i) sum += wave_part[i];
            atomicAdd(&out[span_index], sum);
        }
        __syncthreads();
        acc = 0;
    };

    for (; t < total; t += gridDim.x) {
        if (t >= next) {                       // workgroup-uniform
            fold(s);
            do { ++s; next = prefix[s + 1]; } while (t >= next);
            first = prefix[s];
            sp = spans[s];
        }
        const u64 off = u64(t - first) * TILE;
        const u64 left = sp.nbytes - off;
        const uint8_t *base = reinterpret_cast<const uint8_t *>(sp.ptr) + off;
        // key of the first word this lane reads in the tile
        u64 key = (off / 8 + 2 * u64(tid)) * kGamma;
        if (left >= TILE) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load16(base + (u64(u) * kThreads + tid) * 16);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u64 k0 = key + u64(u) * (2 * kThreads) * kGamma;
                acc += mix(lohi(v[u].x, v[u].y) ^ k0);
                acc += mix(lohi(v[u].z, v[u].w) ^ (k0 + kGamma));
            }
        } else {
            const u64 nvec = left / 16;
            for (u64 i = tid; i < nvec; i += kThreads) {
                const u32x4 v = load16(base + i * 16);
                acc += mix(lohi(v.x, v.y) ^ key);
                acc += mix(lohi(v.z, v.w) ^ (key + kGamma));
                key += u64(2 * kThreads) * kGamma;
            }
            const u32 rem = u32(left % 16);
            if (rem != 0 && tid == 0) {        // ragged end: at most two partial words
                const uint8_t *p = base + nvec * 16;
                const u64 i0 = off / 8 + 2 * nvec;
                acc += mix(tail_word(p, rem) ^ (i0 * kGamma));
                if (rem > 8) acc += mix(tail_word(p + 8, rem - 8) ^ ((i0 + 1) * kGamma));
            }
        }
    }
    fold(s);
}

// -------------------------------------------------------------------- compare
// differs[s] = 1 if the two extents of pair s differ in any byte.  `differs`
// must be zero before the launch.
template <int U>
__global__ __launch_bounds__(kThreads) void compare_kernel(const Pair *__restrict__ pairs,
                                                            const u32 *__restrict__ prefix,
                                                            u32 n_pairs, u32 *__restrict__ differs) {
    constexpr u64 TILE = tile_bytes<U>();
    const u32 total = prefix[n_pairs];
    const u32 tid = threadIdx.x;
    u32 t = blockIdx.x;
    if (t >= total) return;
    u32 s = locate_first(prefix, n_pairs, t);
    u32 first = prefix[s], next = prefix[s + 1];
    Pair pr = pairs[s];
    u32 diff = 0;

    auto fold = [&](u32 pair_index) {
        if (__any(diff != 0) && (tid & 63) == 0) atomicOr(&differs[pair_index], 1u);
        diff = 0;
    };

    for (; t < total; t += gridDim.x) {
        if (t >= next) {
            fold(s);
            do { ++s; next = prefix[s + 1]; } while (t >= next);
            first = prefix[s];
            pr = pairs[s];
        }
        const u64 off = u64(t - first) * TILE;
        const u64 left = pr.nbytes - off;
        const uint8_t *pa = reinterpret_cast<const uint8_t *>(pr.a) + off;
        const uint8_t *pb = reinterpret_cast<const uint8_t *>(pr.b) + off;
        if (left >= TILE) {
            u32x4 va[U], vb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                va[u] = load16(pa + (u64(u) * kThreads + tid) * 16);
                vb[u] = load16(pb + (u64(u) * kThreads + tid) * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32x4 x = va[u] ^ vb[u];
                diff |= x.x | x.y | x.z | x.w;
            }
        } else {
            const u64 nvec = left / 16;
            for (u64 i = tid; i < nvec; i += kThreads) {
                const u32x4 x = load16(pa + i * 16) ^ load16(pb + i * 16);
                diff |= x.x | x.y | x.z | x.w;
            }
            const u32 rem = u32(left % 16);
            if (tid < rem) diff |= u32(pa[nvec * 16 + tid] ^ pb[nvec * 16 + tid]);
        }
    }
    fold(s);
}

// --------------------------------------------------------------------- gather
// dst[0..nbytes) = src[0..nbytes) for every row of `copies`; destinations do
// not overlap each other or any source.
template <int U>
__global__ __launch_bounds__(kThreads) void gather_kernel(const Copy *__restrict__ copies,
                                                           const u32 *__restrict__ prefix,
                                                           u32 n_copies) {
    constexpr u64 TILE = tile_bytes<U>();
    const u32 total = prefix[n_copies];
    const u32 tid = threadIdx.x;
    u32 t = blockIdx.x;
    if (t >= total) return;
    u32 s = locate_first(prefix, n_copies, t);
    u32 first = prefix[s], next = prefix[s + 1];
    Copy cp = copies[s];

    for (; t < total; t += gridDim.x) {
        if (t >= next) {
            do { ++s; next = prefix[s + 1]; } while (t >= next);
            first = prefix[s];
            cp = copies[s];
        }
        const u64 off = u64(t - first) * TILE;
        const u64 left = cp.nbytes - off;
        const uint8_t *ps = reinterpret_cast<const uint8_t *>(cp.src) + off;
        uint8_t *pd = reinterpret_cast<uint8_t *>(cp.dst) + off;
        if (left >= TILE) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load16(ps + (u64(u) * kThreads + tid) * 16);
#pragma unroll
            for (int u = 0; u < U; ++u) store16(pd + (u64(u) * kThreads + tid) * 16, v[u]);
        } else {
            const u64 nvec = left / 16;
            for (u64 i = tid; i < nvec; i += kThreads) store16(pd + i * 16, load16(ps + i * 16));
            const u32 rem = u32(left % 16);
            if (tid < rem) pd[nvec * 16 + tid] = ps[nvec * 16 + tid];
        }
    }
}

// Sets n 64-bit words to zero (result words of the kernels above).
__global__ void zero_words_kernel(u64 *p, u32 n) {
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace tgk
