// Device kernels of the Load path for gfx950 (CDNA4, wave64).
//
// Three streaming kernels share one work decomposition.  A launch covers a
// table of extents (spans to fingerprint, pairs to compare, copies to make).
// Every extent is cut into tiles of T lanes x 16 bytes x U; the tiles of all
// extents are numbered consecutively and every workgroup takes one contiguous
// run of `run` tiles (workgroup b: tiles [b*run, (b+1)*run)), so each
// workgroup streams through one long address range and changes extent only where
// an extent ends inside its run (fingerprint and compare; the copy hands its
// tiles out one by one, see gather_kernel).  Each lane issues U independent
// 128-bit loads before it consumes any of them.
//
// Measured on MI355X (13.5 GB, 291 extents): dealing tiles round-robin
// instead costs a quarter of the fingerprint's bandwidth (a descriptor fetch
// and a cross-wave fold at almost every tile); two to four workgroups of 256
// lanes per compute unit read equally fast, one starves.  The copy does best
// with 1024-lane workgroups that read a 64 KiB tile, meet at a barrier, then
// write it: keeping a compute unit's reads and writes in separate bursts is
// worth ~10 %, and handing the tiles out dynamically another 12-17 %.
//
// None of this is a dense contraction, so there is no MFMA here; nothing is
// reused across tiles, so the only data kept in LDS are the per-wave partial
// sums of the fingerprint's cross-wave combine and the gather's ticket.  The XCD a workgroup lands on
// does not matter for correctness or reuse (each byte is touched once); the
// descriptor tables are a few KiB and end up in every XCD's L2.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tgk {

typedef unsigned long long u64;
typedef unsigned int u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int kReadThreads = 256;           // fingerprint / compare workgroup: 4 waves
constexpr int kCopyThreads = 1024;          // gather workgroup: 16 waves
constexpr u64 kGamma = 0x9E3779B97F4A7C15ull;

struct Span { u64 ptr, nbytes; };           // extent to fingerprint
struct Pair { u64 a, b, nbytes; };          // extents to compare
// Extent to copy (non-overlapping).  A launch that also fingerprints what it copies adds the sum
// over this extent's words to out[slot], the first word counting as word number word0 of its tensor.
struct Copy { u64 dst, src, nbytes, word0; u32 slot, pad; };

template <int T, int U> constexpr u64 tile_bytes() { return u64(T) * 16 * U; }

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

// Every extent lives in global memory (HBM, or pinned host memory seen through
// its device mapping).  Addresses arrive as integers in descriptor tables, so
// the compiler cannot infer the address space; naming it here turns what
// would be FLAT accesses into GLOBAL ones.
#define TGK_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ u32x4 load16(const void *p) {
    return __builtin_nontemporal_load(
        reinterpret_cast<const TGK_GLOBAL u32x4 *>(reinterpret_cast<uintptr_t>(p)));
}
__device__ __forceinline__ void store16(void *p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<TGK_GLOBAL u32x4 *>(reinterpret_cast<uintptr_t>(p)));
}
__device__ __forceinline__ uint8_t load1(const void *p) {
    return *reinterpret_cast<const TGK_GLOBAL uint8_t *>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ void store1(void *p, uint8_t v) {
    *reinterpret_cast<TGK_GLOBAL uint8_t *>(reinterpret_cast<uintptr_t>(p)) = v;
}

// Little-endian word made of up to 8 bytes at p; bytes at or past `avail` are 0.
__device__ __forceinline__ u64 tail_word(const uint8_t *p, u32 avail) {
    u64 w = 0;
    for (u32 j = 0; j < 8 && j < avail; ++j) w |= u64(load1(p + j)) << (8 * j);
    return w;
}

// Walks the tiles [blockIdx.x * run, (blockIdx.x + 1) * run) of a table.
struct TileWalk {
    u32 t, end, s, first, next;
    __device__ __forceinline__ bool init(const u32 *__restrict__ prefix, u32 n, u32 run) {
        const u32 total = prefix[n];
        const u64 lo = u64(blockIdx.x) * run;
        if (lo >= total) return false;
        t = u32(lo);
        end = u32(lo + run < total ? lo + run : total);
        s = locate_first(prefix, n, t);
        first = prefix[s];
        next = prefix[s + 1];
        return true;
    }
    // true when tile t lies past extent s; moves s to the extent that holds t
    __device__ __forceinline__ bool crossed(const u32 *__restrict__ prefix) {
        if (t < next) return false;
        do { ++s; next = prefix[s + 1]; } while (t >= next);
        first = prefix[s];
        return true;
    }
};

// ---------------------------------------------------------------- fingerprint
// out[s] += sum over the words of span s of mix(w_i ^ i*gamma).  `out` must be
// zero before the launch.  Per-lane sums are carried across the tiles of one
// span and folded (wave DPP reduce, LDS across the waves, one 64-bit atomic per
// workgroup) only when the workgroup's run leaves that span.
template <int T, int U>
__global__ __launch_bounds__(T) void fingerprint_kernel(const Span *__restrict__ spans,
                                                         const u32 *__restrict__ prefix, u32 n_spans,
                                                         u32 run, u64 *__restrict__ out) {
    constexpr u64 TILE = tile_bytes<T, U>();
    __shared__ u64 wave_part[T / 64];
    const u32 tid = threadIdx.x;
    TileWalk w;
    if (!w.init(prefix, n_spans, run)) return;     // workgroup-uniform
    Span sp = spans[w.s];
    u64 acc = 0;

    auto fold = [&](u32 span_index) {
        const u64 ws = wave_sum(acc);
        if ((tid & 63) == 0) wave_part[tid >> 6] = ws;
        __syncthreads();
        if (tid == 0) {
            u64 sum = 0;
#pragma unroll
            for (int i = 0; i < T / 64; ++i) sum += wave_part[i];
            atomicAdd(&out[span_index], sum);
        }
        __syncthreads();
        acc = 0;
    };

    for (; w.t < w.end; ++w.t) {
        const u32 prev = w.s;
        if (w.crossed(prefix)) {                   // workgroup-uniform
            fold(prev);
            sp = spans[w.s];
        }
        const u64 off = u64(w.t - w.first) * TILE;
        const u64 left = sp.nbytes - off;
        const uint8_t *base = reinterpret_cast<const uint8_t *>(sp.ptr) + off;
        // key of the first word this lane reads in the tile
        u64 key = (off / 8 + 2 * u64(tid)) * kGamma;
        if (left >= TILE) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load16(base + (u64(u) * T + tid) * 16);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u64 k0 = key + u64(u) * (2 * T) * kGamma;
                acc += mix(lohi(v[u].x, v[u].y) ^ k0);
                acc += mix(lohi(v[u].z, v[u].w) ^ (k0 + kGamma));
            }
        } else {
            const u64 nvec = left / 16;
            for (u64 i = tid; i < nvec; i += T) {
                const u32x4 v = load16(base + i * 16);
                acc += mix(lohi(v.x, v.y) ^ key);
                acc += mix(lohi(v.z, v.w) ^ (key + kGamma));
                key += u64(2 * T) * kGamma;
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
    fold(w.s);
}

// -------------------------------------------------------------------- compare
// differs[s] = 1 if the two extents of pair s differ in any byte.  `differs`
// must be zero before the launch.
template <int T, int U>
__global__ __launch_bounds__(T) void compare_kernel(const Pair *__restrict__ pairs,
                                                     const u32 *__restrict__ prefix, u32 n_pairs,
                                                     u32 run, u32 *__restrict__ differs) {
    constexpr u64 TILE = tile_bytes<T, U>();
    const u32 tid = threadIdx.x;
    TileWalk w;
    if (!w.init(prefix, n_pairs, run)) return;
    Pair pr = pairs[w.s];
    u32 diff = 0;

    auto fold = [&](u32 pair_index) {
        if (__any(diff != 0) && (tid & 63) == 0) atomicOr(&differs[pair_index], 1u);
        diff = 0;
    };

    for (; w.t < w.end; ++w.t) {
        const u32 prev = w.s;
        if (w.crossed(prefix)) {
            fold(prev);
            pr = pairs[w.s];
        }
        const u64 off = u64(w.t - w.first) * TILE;
        const u64 left = pr.nbytes - off;
        const uint8_t *pa = reinterpret_cast<const uint8_t *>(pr.a) + off;
        const uint8_t *pb = reinterpret_cast<const uint8_t *>(pr.b) + off;
        if (left >= TILE) {
            u32x4 va[U], vb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                va[u] = load16(pa + (u64(u) * T + tid) * 16);
                vb[u] = load16(pb + (u64(u) * T + tid) * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32x4 x = va[u] ^ vb[u];
                diff |= x.x | x.y | x.z | x.w;
            }
        } else {
            const u64 nvec = left / 16;
            for (u64 i = tid; i < nvec; i += T) {
                const u32x4 x = load16(pa + i * 16) ^ load16(pb + i * 16);
                diff |= x.x | x.y | x.z | x.w;
            }
            const u32 rem = u32(left % 16);
            if (tid < rem) diff |= u32(load1(pa + nvec * 16 + tid) ^ load1(pb + nvec * 16 + tid));
        }
    }
    fold(w.s);
}

// --------------------------------------------------------------------- gather
// dst[0..nbytes) = src[0..nbytes) for every row of `copies`; destinations do
// not overlap each other or any source.  The workgroup reads a whole tile,
// meets at a barrier, then writes it, so that its loads and its stores reach
// memory as two bursts rather than interleaved.
//
// Tiles are handed out one at a time through `ticket` (a counter that is zero
// before the launch): a workgroup that is done takes the next tile, whichever
// extent it belongs to.  Workgroups do not run at the same pace -- with equal
// contiguous runs the fast ones wait for the slow ones at the end, which costs
// a copy 12-17 % on MI355X (5.93 against 6.65-6.97 TB/s over 7 GiB).  The
// ticket is drawn at the top of the loop and waited for; drawing the next one
// while the current tile is being stored measured 2 % slower.  Unlike the
// fingerprint, a copy carries nothing from tile to tile, so changing extent
// costs one table look-up.
//
// With FP the launch also fingerprints every extent as it passes through the
// registers (out[slot] += the sum over the extent's words; it vouches for the
// bytes that were read).  A tile's arithmetic is put off by one turn of the
// loop: it runs right after the loads of the next tile have been issued, so the
// integer units work while those loads and the previous stores are in flight
// instead of holding up the next loads.  The wave sums meet in LDS; at the top
// of the next turn the first lane of the second wave adds them up while the
// first lane of the first wave draws the ticket.  Both of these lone-lane
// blocks stand together at the top of the loop, before its first barrier: with
// one at the end of the loop body and one at its top the compiler threaded the
// lane from the first straight into the second, across the back edge, and the
// barriers were no longer reached by the whole workgroup in step.
template <int T, int U, bool FP>
__global__ __launch_bounds__(T) void gather_kernel(const Copy *__restrict__ copies,
                                                    const u32 *__restrict__ prefix, u32 n_copies,
                                                    u32 *__restrict__ ticket, u64 *__restrict__ out) {
    constexpr u64 TILE = tile_bytes<T, U>();
    constexpr u32 VPT = u32(T) * U;                // 16-byte vectors per tile
    __shared__ u32 next_tile;
    __shared__ u64 wave_part[T / 64];
    const u32 tid = threadIdx.x;
    const u32 total = prefix[n_copies];
    // FP: the tile of the previous turn, still in registers, and what its sum belongs to
    u32x4 a[U];
    u64 a_key = 0, a_extra = 0;
    u32 a_nvec = 0, a_slot = 0;
    bool have_a = false;
    // FP: wave sums waiting in wave_part for lane 0
    bool pending = false;
    u32 pending_slot = 0;
    for (;;) {
        if (FP && pending && tid == 64) {          // the second wave adds up the sums while the first draws
            u64 sum = 0;
#pragma unroll
            for (int i = 0; i < T / 64; ++i) sum += wave_part[i];
            atomicAdd(&out[pending_slot], sum);
        }
        if (tid == 0) next_tile = atomicAdd(ticket, 1u);
        pending = false;
        __syncthreads();
        const u32 t = __builtin_amdgcn_readfirstlane(next_tile);
        __syncthreads();                           // every lane has read next_tile
        const bool more = t < total;               // workgroup-uniform
        u32x4 b[U];
        u64 b_key = 0, b_extra = 0;
        u32 b_nvec = 0, b_slot = 0;
        uint8_t *pd = nullptr;
        if (more) {
            const u32 s = locate_first(prefix, n_copies, t);
            const Copy cp = copies[s];
            const u64 off = u64(t - prefix[s]) * TILE;
            const u64 left = cp.nbytes - off;
            const uint8_t *ps = reinterpret_cast<const uint8_t *>(cp.src) + off;
            pd = reinterpret_cast<uint8_t *>(cp.dst) + off;
            if (left >= TILE) {                    // workgroup-uniform
                b_nvec = VPT;
#pragma unroll
                for (int u = 0; u < U; ++u) b[u] = load16(ps + (u64(u) * T + tid) * 16);
            } else {
                b_nvec = u32(left / 16);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const u32 i = u32(u) * T + tid;
                    b[u] = i < b_nvec ? load16(ps + u64(i) * 16) : u32x4{0, 0, 0, 0};
                }
                const u32 rem = u32(left % 16);    // ragged end of the extent: single bytes
                if (tid < rem) store1(pd + u64(b_nvec) * 16 + tid, load1(ps + u64(b_nvec) * 16 + tid));
                if (FP && rem != 0 && tid == 0) {  // at most two partial words
                    const uint8_t *p = ps + u64(b_nvec) * 16;
                    const u64 i0 = cp.word0 + off / 8 + 2 * u64(b_nvec);
                    b_extra = mix(tail_word(p, rem) ^ (i0 * kGamma));
                    if (rem > 8) b_extra += mix(tail_word(p + 8, rem - 8) ^ ((i0 + 1) * kGamma));
                }
            }
            if (FP) {
                b_key = (cp.word0 + off / 8 + 2 * u64(tid)) * kGamma;
                b_slot = cp.slot;
            }
        }
        if (FP && have_a) {                        // the previous tile's sum, while this tile's loads fly
            u64 acc = a_extra;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u32(u) * T + tid < a_nvec) {
                    const u64 k0 = a_key + u64(u) * (2 * T) * kGamma;
                    acc += mix(lohi(a[u].x, a[u].y) ^ k0);
                    acc += mix(lohi(a[u].z, a[u].w) ^ (k0 + kGamma));
                }
            }
            const u64 ws = wave_sum(acc);
            if ((tid & 63) == 0) wave_part[tid >> 6] = ws;
            pending = true;
            pending_slot = a_slot;
            have_a = false;
        }
        __syncthreads();                           // the workgroup's loads are all issued; wave_part is complete
        if (!more) {
            if (FP && pending && tid == 0) {
                u64 sum = 0;
#pragma unroll
                for (int i = 0; i < T / 64; ++i) sum += wave_part[i];
                atomicAdd(&out[pending_slot], sum);
            }
            return;
        }
        if (b_nvec == VPT) {
#pragma unroll
            for (int u = 0; u < U; ++u) store16(pd + (u64(u) * T + tid) * 16, b[u]);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32 i = u32(u) * T + tid;
                if (i < b_nvec) store16(pd + u64(i) * 16, b[u]);
            }
        }
        if (FP) {
#pragma unroll
            for (int u = 0; u < U; ++u) a[u] = b[u];
            a_key = b_key;
            a_extra = b_extra;
            a_nvec = b_nvec;
            a_slot = b_slot;
            have_a = true;
        }
        __syncthreads();                           // the next tile's loads start after this tile's stores
    }
}

// ------------------------------------------------------------------ mix rate
// The fingerprint's arithmetic without its loads: every lane mixes
// iters x 16 words that it makes up in registers (key and word advance by
// constants, as in the tiles' inner loop).  Measures the integer-ALU limit of
// the fingerprint; the sum is stored only if it hits one particular value, so
// the work cannot be optimised away and nothing is written in practice.
template <int T>
__global__ __launch_bounds__(T) void mix_rate_kernel(u64 *__restrict__ sink, u32 iters, u64 seed) {
    const u64 lane = u64(blockIdx.x) * T + threadIdx.x;
    u64 key = lane * kGamma, w = seed ^ (lane << 17), acc = 0;
    for (u32 it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            acc += mix(w ^ key);
            key += kGamma;
            w += 0x0123456789ABCDEFull;
        }
    }
    if (acc == 0x5DEECE66D1CE4E5Bull) sink[0] = acc;
}

// Sets n 64-bit words to zero (result words of the kernels above).
__global__ void zero_words_kernel(u64 *p, u32 n) {
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace tgk
