// C ABI of the Load path (see include/tangram.h): argument checks, descriptor
// tables, kernel launches, the host-to-device side stream and commit.
#include "../../include/tangram.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hip.h"
#include "reuse_store.h"

namespace {

using tgk::u32;
using tgk::u64;

#define TG_HIP(call) do { if ((call) != hipSuccess) { (void)hipGetLastError(); return TG_ERR_HIP; } } while (0)

// Loads in flight per lane (U) and resident workgroups per compute unit for
// each kernel, the size up to which a missing tensor rides in the gather launch,
// the copy-grouping threshold (0: none), and whether a verifying load fingerprints
// copied tensors inside the copy launch.  Chosen by measurement on MI355X.
constexpr tg_tuning kDefaultTuning = {8, 4, 4, 1, 4, 2, uint64_t(64) << 10, 0, 1, 0};

// A move whose source and destination overlap goes through this much staging at a time.
constexpr size_t kBounceBytes = size_t(128) << 20;
// A stretch of moves whose first byte shifts by at least this much is copied
// straight (up to that many bytes per launch); below it launches would be too
// small to be worth their launch cost and the stretch is staged.
constexpr uint64_t kDirectShift = uint64_t(32) << 20;

// A verifying load cuts the host-to-device copies of a feed into this many
// batches and fingerprints each as soon as it has landed.
constexpr size_t kVerifyBatches = 4;
// ... but only batches of at least this many bytes: a dependency between two
// streams costs far more than a small copy (measured: a 9 MB model loads in
// 0.16 ms when the host joins the streams and in 1.4 ms with four event waits).
constexpr uint64_t kVerifyBatchMinBytes = uint64_t(64) << 20;

// Library-owned device resources of one owner (a pool, or the calls that take
// no pool): one pinned and one device buffer that hold descriptor tables, tile
// prefixes and result words, the staging buffer of merge moves, and events.
struct DeviceTables {
    void *h = nullptr, *d = nullptr;
    size_t cap = 0;
    int cu_count = 0;
    int device = -1;                    // the device these resources live on
    std::vector<hipEvent_t> events;
    void *bounce = nullptr;             // staging for moves whose source and destination overlap

    tg_status init() {
        int dev = 0;
        TG_HIP(hipGetDevice(&dev));
        if (cu_count != 0) return dev == device ? TG_OK : TG_ERR_INVALID;
        int cus = 0;
        TG_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        cu_count = cus > 0 ? cus : 256;
        device = dev;
        return TG_OK;
    }
    // Room for `bytes` of tables.  Only called while nothing that reads the
    // tables is in flight: growing replaces the buffers.
    tg_status ensure(size_t bytes) {
        const tg_status rc = init();
        if (rc != TG_OK) return rc;
        if (bytes <= cap) return TG_OK;
        size_t want = std::max<size_t>(bytes * 2, size_t(1) << 20);
        release_buffers();
        if (hipHostMalloc(&h, want, hipHostMallocDefault) != hipSuccess) { h = nullptr; (void)hipGetLastError(); return TG_ERR_NOMEM; }
        if (hipMalloc(&d, want) != hipSuccess) { (void)hipHostFree(h); h = d = nullptr; (void)hipGetLastError(); return TG_ERR_NOMEM; }
        cap = want;
        return TG_OK;
    }
    void release_buffers() {
        if (h) (void)hipHostFree(h);
        if (d) (void)hipFree(d);
        h = d = nullptr;
        cap = 0;
    }
    tg_status ensure_bounce() {
        if (bounce) return TG_OK;
        if (hipMalloc(&bounce, kBounceBytes) != hipSuccess) { bounce = nullptr; (void)hipGetLastError(); return TG_ERR_NOMEM; }
        return TG_OK;
    }
    // Event number i of this owner, created on first use and kept.
    tg_status event(size_t i, hipEvent_t *out) {
        while (events.size() <= i) {
            hipEvent_t e = nullptr;
            TG_HIP(hipEventCreate(&e));
            try { events.push_back(e); } catch (...) { (void)hipEventDestroy(e); return TG_ERR_NOMEM; }
        }
        *out = events[i];
        return TG_OK;
    }
    void shutdown() {
        release_buffers();
        if (bounce) { (void)hipFree(bounce); bounce = nullptr; }
        for (auto &e : events) if (e) (void)hipEventDestroy(e);
        events.clear();
        cu_count = 0;
        device = -1;
    }
};

// Resources of tg_fingerprint / tg_compare, which take no pool.
struct SharedTables {
    std::mutex mu;
    DeviceTables t;
} g_shared;

}  // namespace

struct Session;

struct tg_pool {
    tg::ReuseStore store;
    tg_tuning tune = kDefaultTuning;
    bool profiling = false;
    DeviceTables dev;
    tg_load_plan *in_flight = nullptr;      // the plan whose load has begun and not ended
    tg_pool(uint64_t b, uint64_t c, uint32_t a) : store(b, c, a) {}
};

struct tg_load_plan {
    tg::Plan plan;
    std::vector<tg_plan_op> rows;
    std::vector<tg_move> move_rows;
    tg_timing timing = {};
    tg_pool *pool = nullptr;
    Session *session = nullptr;             // between begin and the end of the load
};

namespace {

size_t align_up(size_t n, size_t a) { return (n + a - 1) / a * a; }

tgk::Copy copy_row(u64 dst, u64 src, u64 nbytes) { return tgk::Copy{dst, src, nbytes, 0, 0, 0}; }

// Layout of one launch's table inside the scratch buffers.
struct TableLayout {
    size_t desc_off, prefix_off, result_off, total;
};
TableLayout table_layout(size_t n, size_t desc_size, size_t result_size) {
    TableLayout L;
    L.desc_off = 0;
    L.prefix_off = align_up(n * desc_size, 256);
    L.result_off = L.prefix_off + align_up((n + 1) * sizeof(u32), 256);
    L.total = L.result_off + align_up(n * result_size, 256);
    return L;
}

// prefix[s] = number of tiles before extent s.  False if the count overflows.
bool fill_prefix(u32 *prefix, const u64 *nbytes, size_t stride_words, size_t n, u64 tile) {
    u64 acc = 0;
    for (size_t s = 0; s < n; ++s) {
        prefix[s] = u32(acc);
        const u64 nb = nbytes[s * stride_words];
        acc += nb / tile + (nb % tile != 0 ? 1 : 0);          // no wrap for lengths near 2^64
        if (acc >= (u64(1) << 32) - 1) return false;
    }
    prefix[n] = u32(acc);
    return true;
}

u32 grid_for(int cu_count, u32 total_tiles, u32 wgs_per_cu) {
    const u64 resident = u64(cu_count) * std::max<u32>(1, wgs_per_cu);
    return u32(std::max<u64>(1, std::min<u64>(total_tiles, resident)));
}

u32 pick_u(u32 u) { return u >= 16 ? 16 : u >= 8 ? 8 : u >= 4 ? 4 : 2; }

#define TG_FOR_U(U, ...)                                      \
    switch (U) {                                              \
        case 16: { constexpr int kU = 16; __VA_ARGS__; break; } \
        case 8:  { constexpr int kU = 8;  __VA_ARGS__; break; } \
        case 4:  { constexpr int kU = 4;  __VA_ARGS__; break; } \
        default: { constexpr int kU = 2;  __VA_ARGS__; break; } \
    }

u64 tile_for(u32 threads, u32 U) { return u64(threads) * 16 * U; }

// Tiles per workgroup when `total` tiles are split into equal contiguous runs.
u32 run_for(u32 total_tiles, u32 grid) { return (total_tiles + grid - 1) / grid; }

// Waits for a stream when a call leaves early with work still enqueued, so that
// the scratch tables are never reused (or freed) under a running kernel.
struct DrainOnExit {
    hipStream_t st;
    bool armed = true;
    explicit DrainOnExit(hipStream_t s) : st(s) {}
    ~DrainOnExit() { if (armed) { (void)hipStreamSynchronize(st); (void)hipGetLastError(); } }
};

// One fingerprint launch over a span table that is already on the device.
tg_status launch_fingerprint(const DeviceTables &T, const tg_tuning &tune, size_t desc_off, size_t prefix_off,
                             size_t result_off, u32 n, u32 tiles, hipStream_t st) {
    if (tiles == 0) return TG_OK;
    const u32 U = pick_u(tune.fingerprint_unroll);
    char *d = static_cast<char *>(T.d);
    const u32 grid = grid_for(T.cu_count, tiles, tune.fingerprint_wgs_per_cu);
    const u32 run = run_for(tiles, grid);
    TG_FOR_U(U, tgk::fingerprint_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
                    reinterpret_cast<const tgk::Span *>(d + desc_off), reinterpret_cast<const u32 *>(d + prefix_off),
                    n, run, reinterpret_cast<u64 *>(d + result_off)));
    TG_HIP(hipGetLastError());
    return TG_OK;
}

// ---- fingerprint over device-visible spans, with tables T (the caller holds
// whatever lock protects them)
tg_status fingerprint_run(DeviceTables &T, const tg_tuning &tune, const tg_span *spans, u32 n, uint64_t *out_fp,
                          hipStream_t st, float *ms_out) {
    const u32 U = pick_u(tune.fingerprint_unroll);
    const TableLayout L = table_layout(n, sizeof(tgk::Span), sizeof(u64));
    tg_status rc = T.ensure(L.total);
    if (rc != TG_OK) return rc;
    char *h = static_cast<char *>(T.h), *d = static_cast<char *>(T.d);
    tgk::Span *hs = reinterpret_cast<tgk::Span *>(h + L.desc_off);
    for (u32 i = 0; i < n; ++i) {
        hs[i].ptr = u64(reinterpret_cast<uintptr_t>(spans[i].ptr));
        hs[i].nbytes = spans[i].nbytes;
    }
    u32 *hp = reinterpret_cast<u32 *>(h + L.prefix_off);
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Span) / 8, n, tile_for(tgk::kReadThreads, U))) return TG_ERR_INVALID;
    const u32 total_tiles = hp[n];
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ms_out) {
        if ((rc = T.event(0, &e0)) != TG_OK || (rc = T.event(1, &e1)) != TG_OK) return rc;
    }
    u64 *d_out = reinterpret_cast<u64 *>(d + L.result_off);
    u64 *h_out = reinterpret_cast<u64 *>(h + L.result_off);
    DrainOnExit drain(st);
    TG_HIP(hipMemcpyAsync(d, h, L.result_off, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(tgk::zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, st, d_out, n);
    if (ms_out && total_tiles > 0) TG_HIP(hipEventRecord(e0, st));
    rc = launch_fingerprint(T, tune, L.desc_off, L.prefix_off, L.result_off, n, total_tiles, st);
    if (rc != TG_OK) return rc;
    if (ms_out && total_tiles > 0) TG_HIP(hipEventRecord(e1, st));
    TG_HIP(hipMemcpyAsync(h_out, d_out, n * sizeof(u64), hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    if (ms_out) {
        float ms = 0.f;
        if (total_tiles > 0) TG_HIP(hipEventElapsedTime(&ms, e0, e1));
        *ms_out = ms;
    }
    std::memcpy(out_fp, h_out, n * sizeof(u64));
    return TG_OK;
}

tg_status compare_run(DeviceTables &T, const tg_tuning &tune, const tg_pair *pairs, u32 n, uint32_t *out_differs,
                      hipStream_t st, float *ms_out) {
    const u32 U = pick_u(tune.compare_unroll);
    const TableLayout L = table_layout(n, sizeof(tgk::Pair), sizeof(u64));
    tg_status rc = T.ensure(L.total);
    if (rc != TG_OK) return rc;
    char *h = static_cast<char *>(T.h), *d = static_cast<char *>(T.d);
    tgk::Pair *hs = reinterpret_cast<tgk::Pair *>(h + L.desc_off);
    for (u32 i = 0; i < n; ++i) {
        hs[i].a = u64(reinterpret_cast<uintptr_t>(pairs[i].a));
        hs[i].b = u64(reinterpret_cast<uintptr_t>(pairs[i].b));
        hs[i].nbytes = pairs[i].nbytes;
    }
    u32 *hp = reinterpret_cast<u32 *>(h + L.prefix_off);
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Pair) / 8, n, tile_for(tgk::kReadThreads, U))) return TG_ERR_INVALID;
    const u32 total_tiles = hp[n];
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ms_out) {
        if ((rc = T.event(0, &e0)) != TG_OK || (rc = T.event(1, &e1)) != TG_OK) return rc;
    }
    // results are 32-bit flags; the zero kernel clears whole 64-bit words
    u32 *d_out = reinterpret_cast<u32 *>(d + L.result_off);
    u32 *h_out = reinterpret_cast<u32 *>(h + L.result_off);
    DrainOnExit drain(st);
    TG_HIP(hipMemcpyAsync(d, h, L.result_off, hipMemcpyHostToDevice, st));
    const u32 words = (n + 1) / 2;
    hipLaunchKernelGGL(tgk::zero_words_kernel, dim3((words + 255) / 256), dim3(256), 0, st,
                       reinterpret_cast<u64 *>(d_out), words);
    if (total_tiles > 0) {
        const u32 grid = grid_for(T.cu_count, total_tiles, tune.compare_wgs_per_cu);
        if (ms_out) TG_HIP(hipEventRecord(e0, st));
        const u32 run = run_for(total_tiles, grid);
        TG_FOR_U(U, tgk::compare_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
                        reinterpret_cast<const tgk::Pair *>(d + L.desc_off),
                        reinterpret_cast<const u32 *>(d + L.prefix_off), n, run, d_out));
        TG_HIP(hipGetLastError());
        if (ms_out) TG_HIP(hipEventRecord(e1, st));
    }
    TG_HIP(hipMemcpyAsync(h_out, d_out, n * sizeof(u32), hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    if (ms_out) {
        float ms = 0.f;
        if (total_tiles > 0) TG_HIP(hipEventElapsedTime(&ms, e0, e1));
        *ms_out = ms;
    }
    std::memcpy(out_differs, h_out, n * sizeof(u32));
    return TG_OK;
}

// ---- scratch of the entry point that allocates nothing (tg_fingerprint_noalloc)
//
// One array per GPU, part of the code object, so it exists from the moment the
// library is loaded on a device until the process ends.  In host code its name
// is only a stand-in for the symbol: the device address is asked for once per
// device (static_scratch_for) and only that address is handed to kernels and
// copies.  Layout of a launch inside it: TableLayout, as in the growing scratch.
constexpr size_t kStaticScratchBytes = size_t(128) << 10;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
struct StaticScratch {
    std::mutex mu;                               // one call at a time: the table below is shared
    unsigned char *dev[kMaxDevices] = {};        // device address of `scratch`, per device
    int cu_count[kMaxDevices] = {};
    alignas(256) unsigned char host[kStaticScratchBytes];   // the table as it is uploaded, results as they come back
} g_static;

// Address of this device's copy of `scratch` and its compute-unit count; asked
// for at the first call on each device, with that device current.
tg_status static_scratch_for(int device, unsigned char **ptr, int *cus) {
    if (device < 0 || device >= kMaxDevices) return TG_ERR_INVALID;
    if (!g_static.dev[device]) {
        void *p = nullptr;
        TG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return TG_ERR_HIP;
        int n = 0;
        TG_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device));
        g_static.cu_count[device] = n > 0 ? n : 256;
        g_static.dev[device] = static_cast<unsigned char *>(p);
    }
    *ptr = g_static.dev[device];
    *cus = g_static.cu_count[device];
    return TG_OK;
}

// Merge moves as copy launches (Section 3.2, Stage 2).  Moves arrive in
// execution order: ascending addresses, each shifting its tensor towards lower
// addresses inside its own subspace.  Seen as one stream of bytes, a byte's
// destination lies below its source, and below the source of every later byte,
// so launches that run one after the other on a stream never overwrite bytes
// that are still to be read.  Inside one launch reads and writes are
// concurrent, so every destination must lie below the first source the launch
// reads: a stretch whose first byte shifts by d can be copied straight, up to d
// bytes per launch.  When d is small the stretch is staged instead: one launch
// gathers up to kBounceBytes into the staging buffer, the next writes them out.
//
// Every row remembers which move it is a piece of (slot) and where the piece
// starts inside the tensor (word0, in 8-byte words; pieces are cut at multiples
// of 16 bytes), so that a launch can fingerprint the pieces into the tensor's
// result word.  lands[l] says whether launch l writes into the pool (every
// byte of every move passes through exactly one such launch).
tg_status build_move_launches(const std::vector<tg::Move> &moves, uint64_t base, u64 bounce,
                              std::vector<std::vector<tgk::Copy>> &launches, std::vector<char> &lands, u64 &traffic) {
    auto piece = [](u64 dst, u64 src, u64 len, size_t move, u64 done) {
        tgk::Copy c = copy_row(dst, src, len);
        c.slot = u32(move);
        c.word0 = done / 8;
        return c;
    };
    traffic = 0;
    size_t i = 0;
    uint64_t done = 0;                      // bytes of moves[i] already scheduled
    while (i < moves.size()) {
        const tg::Move &f = moves[i];
        if (f.new_off >= f.old_off || f.nbytes == 0) return TG_ERR_INVALID;
        const uint64_t src0 = f.old_off + done, dst0 = f.new_off + done;
        std::vector<tgk::Copy> in, out;
        if (src0 - dst0 >= kDirectShift) {
            while (i < moves.size()) {
                const tg::Move &m = moves[i];
                if (m.new_off >= m.old_off || m.nbytes == 0) return TG_ERR_INVALID;
                const uint64_t d = m.new_off + done, s = m.old_off + done, left = m.nbytes - done;
                if (d < dst0 || d >= src0) break;           // would write where this launch reads
                uint64_t len = std::min<uint64_t>(left, src0 - d);
                if (len < left) len &= ~uint64_t(15);
                if (len == 0) break;
                in.push_back(piece(base + d, base + s, len, i, done));
                traffic += 2 * len;
                done += len;
                if (done < m.nbytes) break;                 // cut short: the launch is full
                ++i;
                done = 0;
            }
        } else {
            uint64_t staged = 0;
            while (i < moves.size() && staged < kBounceBytes) {
                const tg::Move &m = moves[i];
                if (m.new_off >= m.old_off || m.nbytes == 0) return TG_ERR_INVALID;
                const uint64_t d = m.new_off + done, s = m.old_off + done, left = m.nbytes - done;
                uint64_t len = std::min<uint64_t>(left, kBounceBytes - staged);
                if (len < left) len &= ~uint64_t(15);
                if (len == 0) break;
                in.push_back(piece(bounce + staged, base + s, len, i, done));
                out.push_back(piece(base + d, bounce + staged, len, i, done));
                staged += (len + 15) & ~uint64_t(15);
                traffic += 4 * len;
                done += len;
                if (done < m.nbytes) break;
                ++i;
                done = 0;
            }
        }
        if (in.empty()) return TG_ERR_INVALID;
        launches.push_back(std::move(in));
        lands.push_back(out.empty() ? 1 : 0);
        if (!out.empty()) {
            launches.push_back(std::move(out));
            lands.push_back(1);
        }
    }
    return TG_OK;
}

// Inside one copy launch reads and writes are concurrent: no destination may
// touch a source of the same launch, and every extent lies in the pool or in
// the staging buffer.  A mistake in the cutting above then comes back as an
// error code instead of moved tensors that overwrote each other.
tg_status check_move_launches(const std::vector<std::vector<tgk::Copy>> &launches, uint64_t base, uint64_t cap,
                              u64 bounce) {
    auto inside = [&](u64 a, u64 n) {
        const bool in_pool = a >= base && n <= cap && a - base <= cap - n;
        const bool in_bounce = bounce != 0 && a >= bounce && n <= kBounceBytes && a - bounce <= kBounceBytes - n;
        return in_pool || in_bounce;
    };
    std::vector<std::pair<u64, u64>> src, dst;
    for (const auto &launch : launches) {
        src.clear();
        dst.clear();
        for (const tgk::Copy &c : launch) {
            if (c.nbytes == 0 || !inside(c.src, c.nbytes) || !inside(c.dst, c.nbytes)) return TG_ERR_INVALID;
            src.push_back({c.src, c.src + c.nbytes});
            dst.push_back({c.dst, c.dst + c.nbytes});
        }
        std::sort(src.begin(), src.end());
        std::sort(dst.begin(), dst.end());
        for (size_t i = 1; i < dst.size(); ++i)
            if (dst[i].first < dst[i - 1].second) return TG_ERR_INVALID;
        size_t j = 0;
        for (const auto &d : dst) {
            while (j < src.size() && src[j].second <= d.first) ++j;
            // sources are not disjoint in general (none overlap here, but do not rely on it):
            // look at every source that starts before this destination ends
            for (size_t k = j; k < src.size() && src[k].first < d.second; ++k)
                if (src[k].second > d.first) return TG_ERR_INVALID;
        }
    }
    return TG_OK;
}

// Last check before anything is enqueued: every extent a kernel or the copy
// engine will touch lies inside the pool (or the model's host image), and no
// two destinations overlap.  A planner bug then comes back as an error code
// instead of a stray write.
tg_status validate_plan(const tg::Plan &pl, const tg::ReuseStore &store) {
    const uint64_t cap = store.capacity();
    std::vector<std::pair<uint64_t, uint64_t>> dst;        // [begin, end) of every write
    for (size_t k = 0; k < pl.ops.size(); ++k) {
        const tg::Op &op = pl.ops[k];
        if (op.nbytes == 0 || op.dst_off > cap || op.nbytes > cap - op.dst_off) return TG_ERR_INVALID;
        if (op.dst_off % store.align() != 0) return TG_ERR_INVALID;
        if (op.kind == 0) {
            if (op.src_off > cap || op.nbytes > cap - op.src_off) return TG_ERR_INVALID;
            if (pl.alias) {
                if (op.dst_off != op.src_off) return TG_ERR_INVALID;
                continue;                                   // nothing is written
            }
        } else if (pl.host_base && (op.src_off > pl.host_bytes || op.nbytes > pl.host_bytes - op.src_off)) {
            return TG_ERR_INVALID;
        }
        dst.push_back({op.dst_off, op.dst_off + op.nbytes});
    }
    const size_t n_slots = dst.size();                      // the rest of dst: where moved tensors land
    // moved tensors end up where the plan says; new slots may not touch them
    for (const tg::Move &m : pl.moves) {
        if (m.nbytes == 0 || m.old_off > cap || m.nbytes > cap - m.old_off) return TG_ERR_INVALID;
        if (m.new_off >= m.old_off || m.new_off % store.align() != 0) return TG_ERR_INVALID;
        dst.push_back({m.new_off, m.new_off + m.nbytes});
    }
    std::vector<std::pair<uint64_t, uint64_t>> slots(dst.begin(), dst.begin() + n_slots);
    std::sort(dst.begin(), dst.end());
    for (size_t i = 1; i < dst.size(); ++i)
        if (dst[i].first < dst[i - 1].second) return TG_ERR_INVALID;
    // no new slot lies where the gather reads (its sources are where the moves left them)
    if (!pl.alias) {
        std::sort(slots.begin(), slots.end());
        std::vector<std::pair<uint64_t, uint64_t>> src;
        for (const tg::Op &op : pl.ops)
            if (op.kind == 0) src.push_back({op.src_off, op.src_off + op.nbytes});
        std::sort(src.begin(), src.end());
        src.erase(std::unique(src.begin(), src.end()), src.end());
        size_t j = 0;
        for (const auto &d : slots) {
            while (j < src.size() && src[j].second <= d.first) ++j;
            for (size_t k = j; k < src.size() && src[k].first < d.second; ++k)
                if (src[k].second > d.first) return TG_ERR_INVALID;
        }
    }
    return TG_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

tg_status check_model(const tg_model_desc *m, std::vector<tg::TensorIn> &tensors) {
    if (!m || !m->tensors || m->n_tensors == 0 || m->reserved != 0) return TG_ERR_INVALID;
    if (!m->host_base && m->host_bytes != 0) return TG_ERR_INVALID;
    tensors.resize(m->n_tensors);
    for (u32 k = 0; k < m->n_tensors; ++k) {
        const tg_tensor_desc &t = m->tensors[k];
        if (t.nbytes == 0) return TG_ERR_INVALID;
        // without a host image src_off is the caller's own reference and is not checked
        if (m->host_base && (t.src_off > m->host_bytes || t.nbytes > m->host_bytes - t.src_off)) return TG_ERR_INVALID;
        tensors[k] = tg::TensorIn{t.nbytes, t.fp, t.src_off};
    }
    return TG_OK;
}

}  // namespace

// ------------------------------------------------------------------ load session
// The state of one load between its first enqueued work and its commit:
// which tensors have been handed over, where the next table goes inside the
// pool's scratch, which events time or order what.  tg_assemble runs one from
// start to end inside a single call; tg_assemble_begin / _feed / _wait spread
// it over several.
struct Session {
    tg_pool *pool = nullptr;
    tg_load_plan *lp = nullptr;
    hipStream_t sg = nullptr, sh = nullptr, sh2 = nullptr;
    bool dual = false, verify = false, prof = false;
    // tables are placed one after the other inside the pool's scratch; [0, uploaded)
    // of the pinned copy has been sent to the device copy
    size_t used = 0, uploaded = 0, cap = 0;
    size_t results_off = 0;
    u32 results_cap = 0, results_used = 0;
    std::vector<int64_t> result_ref;        // result word -> tensor index, or -1 - (index of a move)
    std::vector<char> fed;                  // per tensor: nothing (more) to hand over
    u32 unfed = 0;
    size_t next_event = 0;
    struct EvPair { hipEvent_t a, b; };
    std::vector<EvPair> verify_ev, h2d_ev;
    EvPair gather_ev{}, move_ev{};
    bool timed_gather = false, timed_moves = false;
    struct Ticket { hipEvent_t transfer, kernel; };   // null: that stream read nothing of the segment
    std::vector<Ticket> tickets;
    u32 copy_no = 0;                        // host-to-device copies issued so far (deals them over two streams)
    tg_timing t = {};
    std::vector<uint64_t> corrupt_moved;    // moved tensors that no longer match their rows
    bool wrote = false;                     // work that writes into the pool has been enqueued
};

namespace {

struct FeedItem { u32 k; const char *src; };            // tensor index, host address of its bytes
struct FpLaunch { size_t desc_off = 0, prefix_off = 0, result_off = 0; u32 n = 0, tiles = 0; u64 bytes = 0; };
struct CopyLaunch { size_t desc_off = 0, prefix_off = 0, ticket_off = 0; u32 n = 0, tiles = 0; bool fused = false; };

char *tab_h(Session &s) { return static_cast<char *>(s.pool->dev.h); }
char *tab_d(Session &s) { return static_cast<char *>(s.pool->dev.d); }

tg_status tab_alloc(Session &s, size_t bytes, size_t *off) {
    const size_t at = align_up(s.used, 256);
    if (at + bytes > s.cap) return TG_ERR_NOMEM;        // the bound computed at begin was wrong
    s.used = at + bytes;
    *off = at;
    return TG_OK;
}

tg_status new_event(Session &s, hipEvent_t *e) { return s.pool->dev.event(s.next_event++, e); }

// Sends what has been written into the pinned tables since the last upload.
tg_status upload_tables(Session &s) {
    if (s.used > s.uploaded)
        TG_HIP(hipMemcpyAsync(tab_d(s) + s.uploaded, tab_h(s) + s.uploaded, s.used - s.uploaded,
                              hipMemcpyHostToDevice, s.sg));
    s.uploaded = s.used;
    return TG_OK;
}

// Table of one copy launch (rows, tile prefix, ticket counter) in the pinned scratch.
tg_status place_copy_launch(Session &s, const std::vector<tgk::Copy> &rows, CopyLaunch &out) {
    const u64 tile = tile_for(tgk::kCopyThreads, pick_u(s.pool->tune.gather_unroll));
    tg_status rc;
    if ((rc = tab_alloc(s, rows.size() * sizeof(tgk::Copy), &out.desc_off)) != TG_OK) return rc;
    if ((rc = tab_alloc(s, (rows.size() + 1) * sizeof(u32), &out.prefix_off)) != TG_OK) return rc;
    if ((rc = tab_alloc(s, 256, &out.ticket_off)) != TG_OK) return rc;
    char *h = tab_h(s);
    std::memcpy(h + out.desc_off, rows.data(), rows.size() * sizeof(tgk::Copy));
    u32 *hp = reinterpret_cast<u32 *>(h + out.prefix_off);
    if (!fill_prefix(hp, &rows[0].nbytes, sizeof(tgk::Copy) / 8, rows.size(), tile)) return TG_ERR_INVALID;
    out.n = u32(rows.size());
    out.tiles = hp[rows.size()];
    std::memset(h + out.ticket_off, 0, 256);            // the launch's tile counter starts at zero
    return TG_OK;
}

tg_status launch_copy(Session &s, const CopyLaunch &c) {
    if (c.tiles == 0) return TG_OK;
    const tg_tuning &tune = s.pool->tune;
    const u32 U = pick_u(tune.gather_unroll);
    char *d = tab_d(s);
    const u32 grid = grid_for(s.pool->dev.cu_count, c.tiles, tune.gather_wgs_per_cu);
    const tgk::Copy *rows = reinterpret_cast<const tgk::Copy *>(d + c.desc_off);
    const u32 *prefix = reinterpret_cast<const u32 *>(d + c.prefix_off);
    u32 *ticket = reinterpret_cast<u32 *>(d + c.ticket_off);
    if (c.fused) {
        u64 *out = reinterpret_cast<u64 *>(d + s.results_off);
        TG_FOR_U(U, tgk::gather_kernel<tgk::kCopyThreads, kU, true><<<dim3(grid), dim3(tgk::kCopyThreads), 0, s.sg>>>(
                        rows, prefix, c.n, ticket, out));
    } else {
        TG_FOR_U(U, tgk::gather_kernel<tgk::kCopyThreads, kU, false><<<dim3(grid), dim3(tgk::kCopyThreads), 0, s.sg>>>(
                        rows, prefix, c.n, ticket, nullptr));
    }
    TG_HIP(hipGetLastError());
    return TG_OK;
}

// Makes a copy launch fingerprint what it copies: row i's sum goes to a result word of its own,
// remembered as tensor ops[i]'s.
tg_status fuse_fingerprints(Session &s, std::vector<tgk::Copy> &rows, const std::vector<u32> &ops) {
    if (s.results_used + rows.size() > s.results_cap) return TG_ERR_NOMEM;
    for (size_t i = 0; i < rows.size(); ++i) {
        rows[i].slot = s.results_used++;
        rows[i].word0 = 0;
        s.result_ref.push_back(int64_t(ops[i]));
        s.t.fused_verify_bytes += rows[i].nbytes;
    }
    return TG_OK;
}

// Span table of one verification launch: the slots of tensors `ops`, or (moved)
// every tensor the plan moves, at its new address.  Result words are handed out
// in order; result_ref remembers whose each is.
tg_status place_verify(Session &s, const std::vector<u32> &ops, bool moved, FpLaunch &out) {
    const tg::Plan &pl = s.lp->plan;
    const size_t rows = moved ? pl.moves.size() : ops.size();
    out = FpLaunch{};
    if (rows == 0) return TG_OK;
    if (s.results_used + rows > s.results_cap) return TG_ERR_NOMEM;
    tg_status rc;
    if ((rc = tab_alloc(s, rows * sizeof(tgk::Span), &out.desc_off)) != TG_OK) return rc;
    if ((rc = tab_alloc(s, (rows + 1) * sizeof(u32), &out.prefix_off)) != TG_OK) return rc;
    const uint64_t base = s.pool->store.base();
    char *h = tab_h(s);
    tgk::Span *hs = reinterpret_cast<tgk::Span *>(h + out.desc_off);
    for (size_t i = 0; i < rows; ++i) {
        hs[i].ptr = base + (moved ? pl.moves[i].new_off : pl.ops[ops[i]].dst_off);
        hs[i].nbytes = moved ? pl.moves[i].nbytes : pl.ops[ops[i]].nbytes;
        out.bytes += hs[i].nbytes;
        s.result_ref.push_back(moved ? -1 - int64_t(i) : int64_t(ops[i]));
    }
    u32 *hp = reinterpret_cast<u32 *>(h + out.prefix_off);
    const u64 fp_tile = tile_for(tgk::kReadThreads, pick_u(s.pool->tune.fingerprint_unroll));
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Span) / 8, rows, fp_tile)) return TG_ERR_INVALID;
    out.n = u32(rows);
    out.tiles = hp[rows];
    out.result_off = s.results_off + size_t(s.results_used) * sizeof(u64);
    s.results_used += u32(rows);
    return TG_OK;
}

tg_status launch_verify(Session &s, const FpLaunch &f) {
    if (f.tiles == 0) return TG_OK;
    Session::EvPair ev{};
    tg_status rc;
    if (s.prof) {
        if ((rc = new_event(s, &ev.a)) != TG_OK || (rc = new_event(s, &ev.b)) != TG_OK) return rc;
        TG_HIP(hipEventRecord(ev.a, s.sg));
    }
    rc = launch_fingerprint(s.pool->dev, s.pool->tune, f.desc_off, f.prefix_off, f.result_off, f.n, f.tiles, s.sg);
    if (rc != TG_OK) return rc;
    if (s.prof) {
        TG_HIP(hipEventRecord(ev.b, s.sg));
        s.verify_ev.push_back(ev);
    }
    s.t.verify_bytes += f.bytes;
    s.t.verify_launches += 1;
    return TG_OK;
}

// Ends a load that cannot go on: nothing of it may still be running when the
// tables are reused, and the Tensor Mapping must describe the pool's bytes.
tg_status session_fail(tg_load_plan *lp, tg_status rc) {
    Session *s = lp->session;
    if (!s) return rc;
    (void)hipStreamSynchronize(s->sg);
    if (s->sh != s->sg) (void)hipStreamSynchronize(s->sh);
    if (s->dual) (void)hipStreamSynchronize(s->sh2);
    (void)hipGetLastError();
    tg::ReuseStore &store = s->pool->store;
    tg::Plan &pl = lp->plan;
    // evicted tensors may have been overwritten and moved ones have moved:
    // record that much (a plan that did neither has only written into free regions)
    if (s->wrote && (!pl.moves.empty() || !pl.evict.empty())) (void)store.abandon(pl);
    store.drop_corrupt(s->corrupt_moved);
    lp->timing = s->t;
    s->pool->in_flight = nullptr;
    lp->session = nullptr;
    delete s;
    return rc;
}

// Host-to-device part of a feed: `items` are missing tensors whose bytes lie at
// items[i].src (pinned).  Those in `small` have already been dealt with by a
// gather launch.  Copies adjacent on both sides (the slot padding included)
// are merged (Section 4 groups adjacent tensors into large copies); a
// verifying load cuts them into batches and fingerprints each on stream A as
// soon as it has landed on stream B.
tg_status feed_transfers(Session &s, const std::vector<FeedItem> &items, bool may_block, hipEvent_t *done) {
    *done = nullptr;
    if (items.empty()) return TG_OK;
    tg::ReuseStore &store = s.pool->store;
    const tg::Plan &pl = s.lp->plan;
    const uint64_t base = store.base();
    const uint64_t group_limit = s.pool->tune.h2d_group_bytes;
    struct H2D { uint64_t dst; const char *src; uint64_t len, padded; std::vector<u32> ops; };
    std::vector<H2D> h2d;
    h2d.reserve(items.size());
    for (const FeedItem &it : items) {
        const tg::Op &op = pl.ops[it.k];
        h2d.push_back(H2D{op.dst_off, it.src, op.nbytes, store.round_up(op.nbytes), {it.k}});
    }
    std::sort(h2d.begin(), h2d.end(), [](const H2D &a, const H2D &b) { return a.dst < b.dst; });
    std::vector<H2D> merged;
    u64 total = 0;
    for (H2D &c : h2d) {
        total += c.len;
        if (!merged.empty()) {
            H2D &m = merged.back();
            if (m.dst + m.padded == c.dst && m.src + m.padded == c.src && (group_limit == 0 || m.len <= group_limit)) {
                m.len = m.padded + c.len;
                m.padded += c.padded;
                m.ops.push_back(c.ops[0]);
                continue;
            }
        }
        merged.push_back(std::move(c));
    }
    // batch_end[j] = index one past the last merged copy of batch j
    std::vector<size_t> batch_end;
    const size_t nb = !s.verify ? 1 : std::max<size_t>(1, std::min<size_t>(
        std::min<size_t>(kVerifyBatches, merged.size()), size_t(total / kVerifyBatchMinBytes)));
    {
        // shares nb : nb-1 : ... : 1, so that little is left to fingerprint when the last copy lands
        const u64 denom = u64(nb) * (nb + 1) / 2;
        u64 acc = 0, cum = nb;
        for (size_t i = 0; i < merged.size(); ++i) {
            acc += merged[i].len;
            const size_t have = batch_end.size();
            if (i + 1 == merged.size() || (have + 1 < nb && acc * denom >= total * cum)) {
                batch_end.push_back(i + 1);
                cum += nb - (have + 1);
            }
        }
    }
    std::vector<FpLaunch> fp(batch_end.size());
    tg_status rc;
    if (s.verify) {
        size_t from = 0;
        std::vector<u32> ops;
        for (size_t j = 0; j < batch_end.size(); ++j) {
            ops.clear();
            for (size_t i = from; i < batch_end[j]; ++i) ops.insert(ops.end(), merged[i].ops.begin(), merged[i].ops.end());
            if ((rc = place_verify(s, ops, false, fp[j])) != TG_OK) return rc;
            from = batch_end[j];
        }
        if ((rc = upload_tables(s)) != TG_OK) return rc;
    }
    Session::EvPair timed{};
    if (s.prof) {
        if ((rc = new_event(s, &timed.a)) != TG_OK || (rc = new_event(s, &timed.b)) != TG_OK) return rc;
        TG_HIP(hipEventRecord(timed.a, s.sh));
    }
    s.wrote = true;
    size_t from = 0;
    bool any2 = false;
    for (size_t j = 0; j < batch_end.size(); ++j) {
        bool used2 = false;
        for (size_t i = from; i < batch_end[j]; ++i) {
            const H2D &c = merged[i];
            const bool second = s.dual && (s.copy_no & 1) != 0;
            TG_HIP(hipMemcpyAsync(reinterpret_cast<void *>(uintptr_t(base + c.dst)), c.src, c.len,
                                  hipMemcpyHostToDevice, second ? s.sh2 : s.sh));
            used2 = used2 || second;
            s.copy_no += 1;
            s.t.h2d_bytes += c.len;
            s.t.h2d_copies += 1;
        }
        any2 = any2 || used2;
        from = batch_end[j];
        if (s.verify) {
            if (s.sh != s.sg && may_block && total < kVerifyBatchMinBytes) {
                TG_HIP(hipStreamSynchronize(s.sh));        // small transfer: the host joins
                if (used2) TG_HIP(hipStreamSynchronize(s.sh2));
            } else if (s.sh != s.sg) {
                hipEvent_t e;
                if ((rc = new_event(s, &e)) != TG_OK) return rc;
                TG_HIP(hipEventRecord(e, s.sh));
                TG_HIP(hipStreamWaitEvent(s.sg, e, 0));
                if (used2) {
                    if ((rc = new_event(s, &e)) != TG_OK) return rc;
                    TG_HIP(hipEventRecord(e, s.sh2));
                    TG_HIP(hipStreamWaitEvent(s.sg, e, 0));
                }
            }
            if ((rc = launch_verify(s, fp[j])) != TG_OK) return rc;
        }
    }
    if (any2) {                                   // stream B's end covers the second stream
        hipEvent_t e;
        if ((rc = new_event(s, &e)) != TG_OK) return rc;
        TG_HIP(hipEventRecord(e, s.sh2));
        TG_HIP(hipStreamWaitEvent(s.sh, e, 0));
    }
    if (s.prof) {
        TG_HIP(hipEventRecord(timed.b, s.sh));
        s.h2d_ev.push_back(timed);
        *done = timed.b;
    } else {
        hipEvent_t e;
        if ((rc = new_event(s, &e)) != TG_OK) return rc;
        TG_HIP(hipEventRecord(e, s.sh));
        *done = e;
    }
    return TG_OK;
}

// Splits the tensors of a feed into those that ride in a gather launch (read
// through the pinned memory's device mapping) and those the copy engine takes.
void split_small(const Session &s, const std::vector<FeedItem> &items, const void *host_base, void *host_dev,
                 std::vector<tgk::Copy> &small_rows, std::vector<u32> &small_ops, std::vector<FeedItem> &dma) {
    const tg::Plan &pl = s.lp->plan;
    const uint64_t base = s.pool->store.base();
    const uint64_t small = s.pool->tune.h2d_kernel_max_bytes;
    for (const FeedItem &it : items) {
        const tg::Op &op = pl.ops[it.k];
        const u64 mapped = u64(uintptr_t(host_dev)) + u64(it.src - static_cast<const char *>(host_base));
        if (host_dev && small > 0 && op.nbytes <= small && (mapped & 15u) == 0) {
            small_rows.push_back(copy_row(base + op.dst_off, mapped, op.nbytes));
            small_ops.push_back(it.k);
        } else {
            dma.push_back(it);
        }
    }
}

size_t first_dma_count(const std::vector<FeedItem> *v) { return v ? v->size() : 0; }

void *device_mapping(const void *pinned) {
    void *dev = nullptr;
    if (!pinned || hipHostGetDevicePointer(&dev, const_cast<void *>(pinned), 0) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return dev;
}

// Starts a load: checks, tables, moves, gather, the fingerprints that need no
// host bytes.  With `image` (the plan's host image) the load is the classic one:
// its small missing tensors ride in the gather launch and `first_dma` receives
// the rest of the missing tensors for the caller to pass to feed_transfers.
tg_status session_begin(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args, bool image,
                        std::vector<FeedItem> *first_dma) {
    if (!pool || !plan || !args) return TG_ERR_INVALID;
    if (args->flags & ~TG_ASSEMBLE_VERIFY) return TG_ERR_INVALID;
    tg::ReuseStore &store = pool->store;
    tg::Plan &pl = plan->plan;
    if (pl.consumed || pl.pool_tag != &store || plan->session || pool->in_flight) return TG_ERR_INVALID;
    if (pl.generation != store.generation()) return TG_ERR_STALE;
    if (store.model_active(pl.model_id)) return TG_ERR_INVALID;
    if (image && pl.transfer_bytes > 0 && !pl.host_base) return TG_ERR_INVALID;
    tg_status rc = validate_plan(pl, store);
    if (rc != TG_OK) return rc;
    if ((rc = pool->dev.init()) != TG_OK) return rc;
    const uint64_t base = store.base();
    const bool verify = (args->flags & TG_ASSEMBLE_VERIFY) != 0;

    // ---- merge moves (Section 3.2, Stage 2), cut into launches whose reads and writes do not meet
    std::vector<std::vector<tgk::Copy>> move_rows;
    std::vector<char> move_lands;
    u64 move_traffic = 0;
    if (!pl.moves.empty()) {
        if ((rc = pool->dev.ensure_bounce()) != TG_OK) return rc;
        const u64 bounce = u64(reinterpret_cast<uintptr_t>(pool->dev.bounce));
        if ((rc = build_move_launches(pl.moves, base, bounce, move_rows, move_lands, move_traffic)) != TG_OK) return rc;
        if ((rc = check_move_launches(move_rows, base, store.capacity(), bounce)) != TG_OK) return rc;
    }

    Session *sp = new (std::nothrow) Session();
    if (!sp) return TG_ERR_NOMEM;
    struct Guard { Session *s; ~Guard() { delete s; } } guard{sp};
    Session &s = *sp;
    s.pool = pool;
    s.lp = plan;
    s.sg = static_cast<hipStream_t>(args->stream_gather);
    s.sh = static_cast<hipStream_t>(args->stream_h2d);
    // The copies may be dealt over two streams: one copy then starts while the other is still
    // running, which hides what a copy costs to start (about 10 us each on one stream).
    s.sh2 = args->use_second_h2d_stream ? static_cast<hipStream_t>(args->stream_h2d_second) : s.sh;
    s.dual = s.sh2 != s.sh && s.sh2 != s.sg && s.sh != s.sg;
    if (!s.dual) s.sh2 = s.sh;
    s.verify = verify;
    s.prof = pool->profiling;
    s.t = plan->timing;                                   // keeps what tg_plan measured
    s.t.gather_ms = s.t.h2d_ms = s.t.verify_ms = s.t.move_ms = 0.f;
    s.t.gather_bytes = s.t.h2d_bytes = s.t.verify_bytes = s.t.move_bytes = s.t.move_traffic_bytes = 0;
    s.t.fused_verify_bytes = 0;
    s.t.h2d_copies = s.t.move_launches = s.t.verify_launches = s.t.feeds = 0;

    // ---- what the gather launch copies, and what is in place once it has run
    const size_t n = pl.ops.size();
    std::vector<tgk::Copy> copies;
    std::vector<u32> copy_ops;                            // tensor of each row of `copies`
    std::vector<u32> group0;                              // in place without a copy: hits of an aliasing plan
    std::vector<FeedItem> missing;
    const bool fuse = verify && (pool->tune.fuse_verify & 1u) != 0;
    // Moved tensors: fingerprinting them inside the launches that land them saves a pass over HBM
    // but lengthens those launches, which every transfer of the load waits for, while a launch of
    // its own runs beside the transfers; so it is a choice of its own and off by default.
    const bool fuse_moves = verify && (pool->tune.fuse_verify & 2u) != 0;
    try {
        s.fed.assign(n, 1);
        for (size_t k = 0; k < n; ++k) {
            const tg::Op &op = pl.ops[k];
            if (op.kind == 0) {
                if (pl.alias || !fuse) group0.push_back(u32(k));
                if (!pl.alias) {
                    copies.push_back(copy_row(base + op.dst_off, base + op.src_off, op.nbytes));
                    copy_ops.push_back(u32(k));
                }
            } else {
                s.fed[k] = 0;
                s.unfed += 1;
                if (image) missing.push_back(FeedItem{u32(k), static_cast<const char *>(pl.host_base) + op.src_off});
            }
        }
        if (image && !missing.empty()) {
            // small missing tensors ride in the gather launch, read through the pinned
            // image's device mapping, instead of one copy-engine call each
            std::vector<u32> small_ops;
            split_small(s, missing, pl.host_base, device_mapping(pl.host_base), copies, small_ops, *first_dma);
            for (u32 k : small_ops) {
                copy_ops.push_back(k);
                if (!fuse) group0.push_back(k);
                s.fed[k] = 1;
                s.unfed -= 1;
            }
        }
    } catch (...) {
        return TG_ERR_NOMEM;
    }
    for (const auto &c : copies) s.t.gather_bytes += c.nbytes;

    // ---- room for every table this load can need (the buffers cannot grow once a kernel reads them)
    // results; the gather's and the moves' tables; two span tables; per missing tensor one
    // feed at worst, each a dozen small tables padded to 256 bytes
    size_t bound = 8192 + (n + pl.moves.size()) * 64 + copies.size() * 48 + (size_t(s.unfed) + first_dma_count(first_dma) + 1) * 4096;
    for (const auto &rows : move_rows) bound += rows.size() * 48 + 1280;
    if ((rc = pool->dev.ensure(bound)) != TG_OK) return rc;
    s.cap = pool->dev.cap;
    if (verify) {
        s.results_cap = u32(n + pl.moves.size());
        if ((rc = tab_alloc(s, size_t(s.results_cap) * sizeof(u64), &s.results_off)) != TG_OK) return rc;
    }
    s.uploaded = s.used;                                  // result words are cleared by a kernel, not uploaded

    std::vector<CopyLaunch> move_launch(move_rows.size());
    CopyLaunch gather;
    FpLaunch fp_moved, fp_group0;
    try {
        if (fuse_moves && !pl.moves.empty()) {
            // the launches that land the moved bytes also fingerprint them: one result word per move
            if (s.results_used + pl.moves.size() > s.results_cap) return TG_ERR_NOMEM;
            const u32 first = s.results_used;
            for (size_t i = 0; i < pl.moves.size(); ++i) {
                s.result_ref.push_back(-1 - int64_t(i));
                s.t.fused_verify_bytes += pl.moves[i].nbytes;
            }
            s.results_used += u32(pl.moves.size());
            for (size_t l = 0; l < move_rows.size(); ++l) {
                if (!move_lands[l]) continue;
                for (tgk::Copy &c : move_rows[l]) c.slot += first;
                move_launch[l].fused = true;
            }
        }
        for (size_t i = 0; i < move_rows.size(); ++i)
            if ((rc = place_copy_launch(s, move_rows[i], move_launch[i])) != TG_OK) return rc;
        if (fuse && !copies.empty()) {
            if ((rc = fuse_fingerprints(s, copies, copy_ops)) != TG_OK) return rc;
            gather.fused = true;
        }
        if (!copies.empty() && (rc = place_copy_launch(s, copies, gather)) != TG_OK) return rc;
        if (verify) {
            if ((rc = place_verify(s, group0, false, fp_group0)) != TG_OK) return rc;
            if (!fuse_moves && !pl.moves.empty() && (rc = place_verify(s, group0, true, fp_moved)) != TG_OK) return rc;
        }
    } catch (...) {
        return TG_ERR_NOMEM;
    }

    // From here on work is enqueued: the session belongs to the plan, and a failure ends it.
    guard.s = nullptr;
    plan->session = sp;
    plan->pool = pool;
    pool->in_flight = plan;
    auto enqueue = [&]() -> tg_status {
        tg_status r;
        if ((r = upload_tables(s)) != TG_OK) return r;
        if (verify && s.results_cap > 0) {
            tgk::zero_words_kernel<<<dim3((s.results_cap + 255) / 256), dim3(256), 0, s.sg>>>(
                reinterpret_cast<u64 *>(tab_d(s) + s.results_off), s.results_cap);
            TG_HIP(hipGetLastError());
        }
        // ---- moves first (stream A); nothing may land in the pool before they are done
        if (!move_launch.empty()) {
            if ((r = new_event(s, &s.move_ev.a)) != TG_OK || (r = new_event(s, &s.move_ev.b)) != TG_OK) return r;
            if (s.prof) TG_HIP(hipEventRecord(s.move_ev.a, s.sg));
            s.wrote = true;
            for (const CopyLaunch &c : move_launch)
                if ((r = launch_copy(s, c)) != TG_OK) return r;
            TG_HIP(hipEventRecord(s.move_ev.b, s.sg));
            if (s.sh != s.sg) TG_HIP(hipStreamWaitEvent(s.sh, s.move_ev.b, 0));
            if (s.dual) TG_HIP(hipStreamWaitEvent(s.sh2, s.move_ev.b, 0));
            s.timed_moves = s.prof;
            s.t.move_bytes = pl.moved_bytes;
            s.t.move_traffic_bytes = move_traffic;
            s.t.move_launches = u32(move_launch.size());
            if (verify && (r = launch_verify(s, fp_moved)) != TG_OK) return r;    // the moved tensors, where they are now
        }
        // ---- gather launch (stream A), then the fingerprint of what it wrote
        if (gather.tiles > 0) {
            if (s.prof) {
                if ((r = new_event(s, &s.gather_ev.a)) != TG_OK || (r = new_event(s, &s.gather_ev.b)) != TG_OK) return r;
                TG_HIP(hipEventRecord(s.gather_ev.a, s.sg));
            }
            s.wrote = true;
            if ((r = launch_copy(s, gather)) != TG_OK) return r;
            if (s.prof) {
                TG_HIP(hipEventRecord(s.gather_ev.b, s.sg));
                s.timed_gather = true;
            }
        }
        if (verify && (r = launch_verify(s, fp_group0)) != TG_OK) return r;
        return TG_OK;
    };
    rc = enqueue();
    if (rc != TG_OK) return session_fail(plan, rc);
    return TG_OK;
}

// One feed of an open load: rows checked by the caller.
tg_status session_feed(Session &s, const void *seg_base, const std::vector<FeedItem> &items, bool small_allowed,
                       bool may_block, uint32_t *ticket) {
    tg_status rc;
    std::vector<tgk::Copy> small_rows;
    std::vector<u32> small_ops;
    std::vector<FeedItem> dma;
    if (small_allowed) split_small(s, items, seg_base, device_mapping(seg_base), small_rows, small_ops, dma);
    else dma = items;
    Session::Ticket tk{nullptr, nullptr};
    if (!small_rows.empty()) {
        CopyLaunch cl;
        FpLaunch fp;
        const bool fuse = s.verify && (s.pool->tune.fuse_verify & 1u) != 0;
        if (fuse) {
            if ((rc = fuse_fingerprints(s, small_rows, small_ops)) != TG_OK) return rc;
            cl.fused = true;
        }
        if ((rc = place_copy_launch(s, small_rows, cl)) != TG_OK) return rc;
        if (s.verify && !fuse && (rc = place_verify(s, small_ops, false, fp)) != TG_OK) return rc;
        if ((rc = upload_tables(s)) != TG_OK) return rc;
        s.wrote = true;
        if ((rc = launch_copy(s, cl)) != TG_OK) return rc;
        if ((rc = new_event(s, &tk.kernel)) != TG_OK) return rc;
        TG_HIP(hipEventRecord(tk.kernel, s.sg));
        if (s.verify && !fuse && (rc = launch_verify(s, fp)) != TG_OK) return rc;
        for (const auto &c : small_rows) s.t.gather_bytes += c.nbytes;
    }
    if ((rc = feed_transfers(s, dma, may_block, &tk.transfer)) != TG_OK) return rc;
    for (const FeedItem &it : items) {
        s.fed[it.k] = 1;
        s.unfed -= 1;
    }
    s.t.feeds += 1;
    s.tickets.push_back(tk);
    if (ticket) *ticket = uint32_t(s.tickets.size() - 1);
    return TG_OK;
}

// Ends a load: join, timings, integrity check, commit.
tg_status session_wait(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs) {
    Session &s = *plan->session;
    tg::ReuseStore &store = pool->store;
    tg::Plan &pl = plan->plan;
    if (s.unfed != 0) return session_fail(plan, TG_ERR_INVALID);
    auto finish = [&]() -> tg_status {
        if (s.verify && s.results_used > 0)
            TG_HIP(hipMemcpyAsync(tab_h(s) + s.results_off, tab_d(s) + s.results_off, size_t(s.results_used) * sizeof(u64),
                                  hipMemcpyDeviceToHost, s.sg));
        // ---- join
        TG_HIP(hipStreamSynchronize(s.sg));
        if (s.sh != s.sg) TG_HIP(hipStreamSynchronize(s.sh));
        if (s.dual) TG_HIP(hipStreamSynchronize(s.sh2));
        if (s.prof) {
            float ms = 0.f;
            if (s.timed_gather) TG_HIP(hipEventElapsedTime(&ms, s.gather_ev.a, s.gather_ev.b));
            s.t.gather_ms = ms;
            ms = 0.f;
            if (s.timed_moves) TG_HIP(hipEventElapsedTime(&ms, s.move_ev.a, s.move_ev.b));
            s.t.move_ms = ms;
            float total = 0.f;
            for (const auto &ev : s.h2d_ev) {
                TG_HIP(hipEventElapsedTime(&ms, ev.a, ev.b));
                total += ms;
            }
            s.t.h2d_ms = total;
            total = 0.f;
            for (const auto &ev : s.verify_ev) {
                TG_HIP(hipEventElapsedTime(&ms, ev.a, ev.b));
                total += ms;
            }
            s.t.verify_ms = total;
        }
        // ---- the integrity check proper: every slot's fingerprint against its descriptor,
        // every moved tensor's against its row of the Tensor Mapping
        if (s.verify) {
            const u64 *res = reinterpret_cast<const u64 *>(tab_h(s) + s.results_off);
            bool good = true;
            for (size_t i = 0; i < s.result_ref.size(); ++i) {
                const int64_t ref = s.result_ref[i];
                if (ref >= 0) {
                    if (res[i] != pl.fps[size_t(ref)]) good = false;
                } else {
                    const tg::Move &m = pl.moves[size_t(-1 - ref)];
                    if (res[i] != m.fp) { s.corrupt_moved.push_back(m.entry); good = false; }
                }
            }
            if (!good) return TG_ERR_CORRUPT;
        }
        return TG_OK;
    };
    tg_status rc = finish();
    if (rc != TG_OK) return session_fail(plan, rc);

    // ---- commit (Section 3.1: update the mapping, return the addresses)
    std::vector<uint64_t> dst;
    const tg::Status cs = store.commit(pl, dst);
    plan->timing = s.t;
    pool->in_flight = nullptr;
    plan->session = nullptr;
    delete &s;
    if (cs != tg::OK) return tg_status(cs);
    if (out_dev_ptrs)
        for (size_t k = 0; k < dst.size(); ++k)
            out_dev_ptrs[k] = reinterpret_cast<void *>(uintptr_t(store.base() + dst[k]));
    return TG_OK;
}

}  // namespace

extern "C" {

tg_status tg_pool_create(void *dev_base, uint64_t capacity, uint32_t align, tg_pool **out) try {
    if (!dev_base || !out || capacity == 0) return TG_ERR_INVALID;
    if (align < 16 || (align & (align - 1)) != 0) return TG_ERR_INVALID;
    const uint64_t base = uint64_t(reinterpret_cast<uintptr_t>(dev_base));
    if (base % align != 0 || capacity % align != 0) return TG_ERR_INVALID;
    if (base + capacity < base) return TG_ERR_INVALID;
    tg_pool *p = new (std::nothrow) tg_pool(base, capacity, align);
    if (!p) return TG_ERR_NOMEM;
    *out = p;
    return TG_OK;
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_pool_destroy(tg_pool *pool) {
    if (!pool) return TG_OK;
    if (pool->in_flight) (void)session_fail(pool->in_flight, TG_ERR_INVALID);
    pool->dev.shutdown();
    delete pool;
    return TG_OK;
}

tg_status tg_pool_stats(const tg_pool *pool, tg_stats *out) {
    if (!pool || !out) return TG_ERR_INVALID;
    const tg::Stats s = pool->store.stats();
    out->capacity = s.capacity;
    out->free_bytes = s.free_bytes;
    out->largest_free = s.largest_free;
    out->n_regions = s.n_regions;
    out->n_free_regions = s.n_free_regions;
    out->n_entries = s.n_entries;
    out->n_active = s.n_active;
    out->generation = s.generation;
    return TG_OK;
}

tg_status tg_pool_regions(const tg_pool *pool, tg_region *out, uint32_t cap, uint32_t *n) {
    if (!pool || !n || (cap > 0 && !out)) return TG_ERR_INVALID;
    const auto &regions = pool->store.region_list().regions();
    uint32_t i = 0;
    for (const auto &r : regions) {
        if (i < cap) out[i] = tg_region{r.first, r.second.len, r.second.free ? 1u : 0u, 0u};
        ++i;
    }
    *n = i;
    return TG_OK;
}

tg_status tg_pool_entries(const tg_pool *pool, tg_entry *out, uint32_t cap, uint32_t *n) try {
    if (!pool || !n || (cap > 0 && !out)) return TG_ERR_INVALID;
    const std::vector<const tg::Entry *> rows = pool->store.entries_by_offset();
    for (size_t i = 0; i < rows.size() && i < cap; ++i)
        out[i] = tg_entry{rows[i]->off, rows[i]->nbytes, rows[i]->fp, uint32_t(rows[i]->owners.size()),
                          rows[i]->active_refs};
    *n = uint32_t(rows.size());
    return TG_OK;
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_default_tuning(tg_tuning *out) {
    if (!out) return TG_ERR_INVALID;
    *out = kDefaultTuning;
    return TG_OK;
}

tg_status tg_pool_set_tuning(tg_pool *pool, const tg_tuning *t) {
    if (!pool || !t || pool->in_flight) return TG_ERR_INVALID;
    pool->tune = *t;
    return TG_OK;
}

tg_status tg_pool_get_tuning(const tg_pool *pool, tg_tuning *out) {
    if (!pool || !out) return TG_ERR_INVALID;
    *out = pool->tune;
    return TG_OK;
}

tg_status tg_pool_set_profiling(tg_pool *pool, int on) {
    if (!pool || pool->in_flight) return TG_ERR_INVALID;
    pool->profiling = on != 0;
    return TG_OK;
}

tg_status tg_fingerprint_ex(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream,
                            const tg_tuning *tuning, float *kernel_ms) {
    if (n == 0) {
        if (kernel_ms) *kernel_ms = 0.f;
        return TG_OK;
    }
    if (!spans || !out_fp) return TG_ERR_INVALID;
    for (u32 i = 0; i < n; ++i) {
        if (spans[i].nbytes != 0 && !spans[i].ptr) return TG_ERR_INVALID;
        if (!aligned16(spans[i].ptr)) return TG_ERR_INVALID;
    }
    std::vector<uint64_t> tmp;
    try { tmp.resize(n); } catch (...) { return TG_ERR_NOMEM; }
    float ms = 0.f;
    std::lock_guard<std::mutex> lock(g_shared.mu);
    const tg_status rc = fingerprint_run(g_shared.t, tuning ? *tuning : kDefaultTuning, spans, n, tmp.data(),
                                         static_cast<hipStream_t>(stream), kernel_ms ? &ms : nullptr);
    if (rc != TG_OK) return rc;
    std::memcpy(out_fp, tmp.data(), n * sizeof(uint64_t));
    if (kernel_ms) *kernel_ms = ms;
    return TG_OK;
}

tg_status tg_fingerprint(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream) {
    return tg_fingerprint_ex(spans, n, out_fp, stream, nullptr, nullptr);
}

// tg_fingerprint for callers that may not allocate: the span table, the tile
// prefix and the result words live in this device's copy of `scratch`, the host
// side of the table in a static array.  No hipMalloc / hipFree / hipHostMalloc,
// no events, no std::vector.
tg_status tg_fingerprint_noalloc(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream) {
    if (n == 0) return TG_OK;
    if (!spans || !out_fp) return TG_ERR_INVALID;
    if (n > TG_NOALLOC_MAX_SPANS) return TG_ERR_INVALID;
    for (u32 i = 0; i < n; ++i) {
        if (spans[i].nbytes != 0 && !spans[i].ptr) return TG_ERR_INVALID;
        if (!aligned16(spans[i].ptr)) return TG_ERR_INVALID;
    }
    const TableLayout L = table_layout(n, sizeof(tgk::Span), sizeof(u64));
    if (L.total > kStaticScratchBytes) return TG_ERR_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int dev = 0;
    TG_HIP(hipGetDevice(&dev));

    std::lock_guard<std::mutex> lock(g_static.mu);
    unsigned char *d = nullptr;
    int cus = 0;
    const tg_status rc = static_scratch_for(dev, &d, &cus);
    if (rc != TG_OK) return rc;
    // launch shape: the library's defaults (the tuning call belongs to the allocating path)
    constexpr int kU = 8;
    constexpr u32 kWgsPerCu = 4;
    unsigned char *h = g_static.host;
    tgk::Span *hs = reinterpret_cast<tgk::Span *>(h + L.desc_off);
    for (u32 i = 0; i < n; ++i) {
        hs[i].ptr = u64(reinterpret_cast<uintptr_t>(spans[i].ptr));
        hs[i].nbytes = spans[i].nbytes;
    }
    u32 *hp = reinterpret_cast<u32 *>(h + L.prefix_off);
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Span) / 8, n, tile_for(tgk::kReadThreads, kU))) return TG_ERR_INVALID;
    const u32 total_tiles = hp[n];
    u64 *d_out = reinterpret_cast<u64 *>(d + L.result_off);
    DrainOnExit drain(st);
    TG_HIP(hipMemcpyAsync(d, h, L.result_off, hipMemcpyHostToDevice, st));
    // the array keeps the last call's results: the words this call adds into start at zero
    hipLaunchKernelGGL(tgk::zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, st, d_out, n);
    if (total_tiles > 0) {
        const u32 grid = u32(std::max<u64>(1, std::min<u64>(total_tiles, u64(cus) * kWgsPerCu)));
        const u32 run = run_for(total_tiles, grid);
        tgk::fingerprint_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
            reinterpret_cast<const tgk::Span *>(d + L.desc_off), reinterpret_cast<const u32 *>(d + L.prefix_off), n,
            run, d_out);
    }
    TG_HIP(hipGetLastError());
    TG_HIP(hipMemcpyAsync(h + L.result_off, d_out, n * sizeof(u64), hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    std::memcpy(out_fp, h + L.result_off, n * sizeof(u64));
    return TG_OK;
}

tg_status tg_compare_ex(const tg_pair *pairs, uint32_t n, uint32_t *out_differs, void *stream,
                        const tg_tuning *tuning, float *kernel_ms) {
    if (n == 0) {
        if (kernel_ms) *kernel_ms = 0.f;
        return TG_OK;
    }
    if (!pairs || !out_differs) return TG_ERR_INVALID;
    for (u32 i = 0; i < n; ++i) {
        if (pairs[i].nbytes != 0 && (!pairs[i].a || !pairs[i].b)) return TG_ERR_INVALID;
        if (!aligned16(pairs[i].a) || !aligned16(pairs[i].b)) return TG_ERR_INVALID;
    }
    std::vector<uint32_t> tmp;
    try { tmp.resize(n); } catch (...) { return TG_ERR_NOMEM; }
    float ms = 0.f;
    std::lock_guard<std::mutex> lock(g_shared.mu);
    const tg_status rc = compare_run(g_shared.t, tuning ? *tuning : kDefaultTuning, pairs, n, tmp.data(),
                                     static_cast<hipStream_t>(stream), kernel_ms ? &ms : nullptr);
    if (rc != TG_OK) return rc;
    std::memcpy(out_differs, tmp.data(), n * sizeof(uint32_t));
    if (kernel_ms) *kernel_ms = ms;
    return TG_OK;
}

tg_status tg_compare(const tg_pair *pairs, uint32_t n, uint32_t *out_differs, void *stream) {
    return tg_compare_ex(pairs, n, out_differs, stream, nullptr, nullptr);
}

static tg_status plan_impl(tg_pool *pool, const tg_model_desc *model, uint32_t flags, void *stream,
                           tg_load_plan **out);

tg_status tg_plan(tg_pool *pool, const tg_model_desc *model, uint32_t flags, void *stream,
                  tg_load_plan **out) {
    try {
        return plan_impl(pool, model, flags, stream, out);
    } catch (...) {                               // a container could not grow; nothing was changed
        return TG_ERR_NOMEM;
    }
}

static tg_status plan_impl(tg_pool *pool, const tg_model_desc *model, uint32_t flags, void *stream,
                           tg_load_plan **out) {
    if (!pool || !out) return TG_ERR_INVALID;
    if (flags & ~(TG_PLAN_CONFIRM | TG_PLAN_EVICT | TG_PLAN_MERGE | TG_PLAN_ALIAS | TG_PLAN_PACK_TEXT | TG_PLAN_CAP_TEXT))
        return TG_ERR_INVALID;
    const auto t0 = std::chrono::steady_clock::now();
    std::vector<tg::TensorIn> tensors;
    tg_status rc = check_model(model, tensors);
    if (rc != TG_OK) return rc;
    tg::ReuseStore &store = pool->store;
    if (store.model_active(model->model_id)) return TG_ERR_INVALID;
    const bool confirm = (flags & TG_PLAN_CONFIRM) != 0;
    if (confirm && (!model->host_base || pool->in_flight)) return TG_ERR_INVALID;

    const size_t n = tensors.size();
    std::vector<uint64_t> hits(n, 0);
    std::vector<std::pair<uint64_t, uint64_t>> cand;      // (offset, entry id), ascending offset
    float compare_ms = 0.f;
    uint64_t compare_bytes = 0;
    if (!confirm) {
        // Section 3.1: a tensor found in the Tensor Mapping is reused.
        for (size_t k = 0; k < n; ++k) {
            store.candidates(tensors[k].fp, tensors[k].nbytes, cand);
            if (!cand.empty()) hits[k] = cand.front().second;
        }
    } else {
        // Every candidate of every tensor is compared with the incoming bytes
        // in one launch; the first candidate (lowest offset) that is equal wins.
        void *host_dev = device_mapping(model->host_base);
        if (!host_dev) return TG_ERR_INVALID;
        std::vector<tg_pair> pairs;
        std::vector<std::pair<size_t, uint64_t>> who;   // (tensor, candidate entry)
        for (size_t k = 0; k < n; ++k) {
            store.candidates(tensors[k].fp, tensors[k].nbytes, cand);
            for (const auto &c : cand) {
                tg_pair p;
                p.a = reinterpret_cast<const void *>(uintptr_t(store.base() + c.first));
                p.b = static_cast<const char *>(host_dev) + tensors[k].src_off;
                p.nbytes = tensors[k].nbytes;
                if (!aligned16(p.b)) return TG_ERR_INVALID;
                pairs.push_back(p);
                who.push_back({k, c.second});
                compare_bytes += p.nbytes;
            }
        }
        if (!pairs.empty()) {
            std::vector<uint32_t> differs(pairs.size());
            rc = compare_run(pool->dev, pool->tune, pairs.data(), u32(pairs.size()), differs.data(),
                             static_cast<hipStream_t>(stream), pool->profiling ? &compare_ms : nullptr);
            if (rc != TG_OK) return rc;
            for (size_t i = 0; i < pairs.size(); ++i)
                if (!differs[i] && hits[who[i].first] == 0) hits[who[i].first] = who[i].second;
        }
    }

    std::unique_ptr<tg_load_plan> owner(new (std::nothrow) tg_load_plan());
    tg_load_plan *lp = owner.get();
    if (!lp) return TG_ERR_NOMEM;
    lp->pool = pool;
    lp->plan.model_id = model->model_id;
    lp->plan.host_base = model->host_base;
    lp->plan.host_bytes = model->host_bytes;
    const tg::Status ps = store.plan(tensors, hits, flags, lp->plan);
    if (ps != tg::OK) return tg_status(ps);
    lp->rows.resize(n);
    for (size_t k = 0; k < n; ++k) {
        const tg::Op &op = lp->plan.ops[k];
        lp->rows[k] = tg_plan_op{op.kind, 0u, op.dst_off, op.src_off, op.nbytes};
    }
    lp->move_rows.resize(lp->plan.moves.size());
    for (size_t i = 0; i < lp->plan.moves.size(); ++i) {
        const tg::Move &m = lp->plan.moves[i];
        lp->move_rows[i] = tg_move{m.old_off, m.new_off, m.nbytes};
    }
    lp->timing.compare_ms = compare_ms;
    lp->timing.compare_bytes = compare_bytes;
    lp->timing.plan_host_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *out = owner.release();
    return TG_OK;
}

tg_status tg_plan_ops(const tg_load_plan *plan, const tg_plan_op **ops, uint32_t *n,
                      uint64_t *reused_bytes, uint64_t *transfer_bytes) {
    if (!plan) return TG_ERR_INVALID;
    if (ops) *ops = plan->rows.data();
    if (n) *n = uint32_t(plan->rows.size());
    if (reused_bytes) *reused_bytes = plan->plan.reused_bytes;
    if (transfer_bytes) *transfer_bytes = plan->plan.transfer_bytes;
    return TG_OK;
}

tg_status tg_plan_info(const tg_load_plan *plan, tg_plan_summary *out) {
    if (!plan || !out) return TG_ERR_INVALID;
    const tg::Plan &p = plan->plan;
    out->n_tensors = uint32_t(p.ops.size());
    out->n_evictions = uint32_t(p.evict.size());
    out->n_moves = uint32_t(p.moves.size());
    out->alias = p.alias ? 1u : 0u;
    out->n_reused = 0;
    for (const tg::Op &op : p.ops) out->n_reused += op.kind == 0 ? 1u : 0u;
    out->reserved = 0;
    out->reused_bytes = p.reused_bytes;
    out->transfer_bytes = p.transfer_bytes;
    out->copy_bytes = p.copy_bytes;
    out->evicted_bytes = p.evicted_bytes;
    out->moved_bytes = p.moved_bytes;
    out->merge_bound = p.merge_bound;
    return TG_OK;
}

tg_status tg_plan_moves(const tg_load_plan *plan, const tg_move **moves, uint32_t *n) {
    if (!plan) return TG_ERR_INVALID;
    if (moves) *moves = plan->move_rows.data();
    if (n) *n = uint32_t(plan->move_rows.size());
    return TG_OK;
}

tg_status tg_plan_evictions(const tg_load_plan *plan, const uint64_t **offsets, uint32_t *n) {
    if (!plan) return TG_ERR_INVALID;
    if (offsets) *offsets = plan->plan.evict_offs.data();
    if (n) *n = uint32_t(plan->plan.evict_offs.size());
    return TG_OK;
}

tg_status tg_plan_timing(const tg_load_plan *plan, tg_timing *out) {
    if (!plan || !out) return TG_ERR_INVALID;
    *out = plan->session ? plan->session->t : plan->timing;
    return TG_OK;
}

void tg_plan_free(tg_load_plan *plan) {
    if (!plan) return;
    if (plan->session) (void)session_fail(plan, TG_ERR_INVALID);
    delete plan;
}

tg_status tg_commit(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs) try {
    if (!pool || !plan || pool->in_flight) return TG_ERR_INVALID;
    std::vector<uint64_t> dst;
    const tg::Status s = pool->store.commit(plan->plan, dst);
    if (s != tg::OK) return tg_status(s);
    if (out_dev_ptrs)
        for (size_t k = 0; k < dst.size(); ++k)
            out_dev_ptrs[k] = reinterpret_cast<void *>(uintptr_t(pool->store.base() + dst[k]));
    return TG_OK;
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_abandon(tg_pool *pool, tg_load_plan *plan) try {
    if (!pool || !plan || pool->in_flight) return TG_ERR_INVALID;
    return tg_status(pool->store.abandon(plan->plan));
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_assemble_begin(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args) {
    try {
        return session_begin(pool, plan, args, false, nullptr);
    } catch (...) {                               // a container could not grow
        return plan && plan->session ? session_fail(plan, TG_ERR_NOMEM) : TG_ERR_NOMEM;
    }
}

// Starts a load from the plan's whole host image.  may_block: the caller is
// about to wait anyway, so a small transfer may be joined by the host.
static tg_status begin_from_image(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args, bool may_block) {
    std::vector<FeedItem> dma;
    tg_status rc = session_begin(pool, plan, args, true, &dma);
    if (rc != TG_OK) return rc;
    if (!dma.empty()) {
        rc = session_feed(*plan->session, plan->plan.host_base, dma, false, may_block, nullptr);
        if (rc != TG_OK) return session_fail(plan, rc);
    }
    return TG_OK;
}

tg_status tg_assemble_async(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args) {
    try {
        return begin_from_image(pool, plan, args, false);
    } catch (...) {
        return plan && plan->session ? session_fail(plan, TG_ERR_NOMEM) : TG_ERR_NOMEM;
    }
}

tg_status tg_assemble_feed(tg_pool *pool, tg_load_plan *plan, const void *seg_base, uint64_t seg_bytes,
                           const tg_feed_row *rows, uint32_t n, uint32_t *ticket) {
    if (!pool || !plan || !plan->session || pool->in_flight != plan) return TG_ERR_INVALID;
    if (n == 0 || !rows || !seg_base) return TG_ERR_INVALID;
    Session &s = *plan->session;
    const tg::Plan &pl = plan->plan;
    std::vector<FeedItem> items;
    std::vector<char> seen;
    try {
        items.reserve(n);
        seen.assign(pl.ops.size(), 0);
    } catch (...) {
        return TG_ERR_NOMEM;
    }
    for (u32 i = 0; i < n; ++i) {
        const tg_feed_row &r = rows[i];
        if (r.reserved != 0 || r.tensor >= pl.ops.size()) return TG_ERR_INVALID;
        const tg::Op &op = pl.ops[r.tensor];
        if (op.kind != 1 || s.fed[r.tensor] || seen[r.tensor]) return TG_ERR_INVALID;
        if (r.seg_off > seg_bytes || op.nbytes > seg_bytes - r.seg_off) return TG_ERR_INVALID;
        seen[r.tensor] = 1;
        items.push_back(FeedItem{r.tensor, static_cast<const char *>(seg_base) + r.seg_off});
    }
    uint32_t tk = 0;
    tg_status rc;
    try {
        rc = session_feed(s, seg_base, items, true, false, &tk);
    } catch (...) {
        rc = TG_ERR_NOMEM;
    }
    if (rc != TG_OK) return session_fail(plan, rc);
    if (ticket) *ticket = tk;
    return TG_OK;
}

tg_status tg_assemble_feed_wait(tg_pool *pool, tg_load_plan *plan, uint32_t ticket) {
    if (!pool || !plan || !plan->session || pool->in_flight != plan) return TG_ERR_INVALID;
    Session &s = *plan->session;
    if (ticket >= s.tickets.size()) return TG_ERR_INVALID;
    const Session::Ticket tk = s.tickets[ticket];
    if (tk.kernel && hipEventSynchronize(tk.kernel) != hipSuccess) return session_fail(plan, TG_ERR_HIP);
    if (tk.transfer && hipEventSynchronize(tk.transfer) != hipSuccess) return session_fail(plan, TG_ERR_HIP);
    return TG_OK;
}

tg_status tg_assemble_wait(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs) {
    if (!pool || !plan || !plan->session || pool->in_flight != plan) return TG_ERR_INVALID;
    try {
        return session_wait(pool, plan, out_dev_ptrs);
    } catch (...) {
        return session_fail(plan, TG_ERR_NOMEM);
    }
}

tg_status tg_assemble_ex(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args, void **out_dev_ptrs) {
    tg_status rc;
    try {
        rc = begin_from_image(pool, plan, args, true);
    } catch (...) {
        rc = plan && plan->session ? session_fail(plan, TG_ERR_NOMEM) : TG_ERR_NOMEM;
    }
    if (rc != TG_OK) return rc;
    return tg_assemble_wait(pool, plan, out_dev_ptrs);
}

tg_status tg_assemble(tg_pool *pool, tg_load_plan *plan, uint32_t flags, void *stream_gather,
                      void *stream_h2d, void **out_dev_ptrs) {
    tg_assemble_args args;
    args.flags = flags;
    args.use_second_h2d_stream = 0;
    args.stream_gather = stream_gather;
    args.stream_h2d = stream_h2d;
    args.stream_h2d_second = nullptr;
    return tg_assemble_ex(pool, plan, &args, out_dev_ptrs);
}

tg_status tg_release(tg_pool *pool, uint64_t model_id, uint32_t flags) try {
    if (!pool || pool->in_flight) return TG_ERR_INVALID;
    return tg_status(pool->store.release(model_id, (flags & TG_RELEASE_EVICT) != 0));
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_set_model_cost(tg_pool *pool, uint64_t model_id, double miss_prob, double load_bw, double alpha) try {
    if (!pool) return TG_ERR_INVALID;
    return tg_status(pool->store.set_model_cost(model_id, miss_prob, load_bw, alpha));
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_reuse_size(const tg_pool *pool, const tg_model_desc *model, double link_bytes_per_s,
                        uint64_t *reuse_bytes, double *est_load_s) try {
    if (!pool || !reuse_bytes) return TG_ERR_INVALID;
    std::vector<tg::TensorIn> tensors;
    const tg_status rc = check_model(model, tensors);
    if (rc != TG_OK) return rc;
    if (est_load_s && !(link_bytes_per_s > 0.0)) return TG_ERR_INVALID;
    const uint64_t reuse = pool->store.reuse_size(tensors);
    uint64_t total = 0;
    for (const auto &t : tensors) total += t.nbytes;
    *reuse_bytes = reuse;
    // Eq. 3: t_load = (S - S') / B
    if (est_load_s) *est_load_s = double(total - reuse) / link_bytes_per_s;
    return TG_OK;
} catch (...) {
    return TG_ERR_NOMEM;                          // a container could not grow
}

tg_status tg_host_alloc(uint64_t nbytes, void **out) {
    if (!out || nbytes == 0) return TG_ERR_INVALID;
    void *p = nullptr;
    if (hipHostMalloc(&p, nbytes, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return TG_ERR_NOMEM;
    }
    *out = p;
    return TG_OK;
}

tg_status tg_host_free(void *p) {
    if (!p) return TG_OK;
    TG_HIP(hipHostFree(p));
    return TG_OK;
}

tg_status tg_measure_mix_rate(uint32_t iters, void *stream, double *words_per_s) {
    if (!words_per_s || iters == 0 || iters > (1u << 20)) return TG_ERR_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_shared.mu);
    DeviceTables &T = g_shared.t;
    tg_status rc = T.ensure(4096);
    if (rc != TG_OK) return rc;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if ((rc = T.event(0, &e0)) != TG_OK || (rc = T.event(1, &e1)) != TG_OK) return rc;
    const u32 grid = u32(T.cu_count) * 8;
    DrainOnExit drain(st);
    TG_HIP(hipEventRecord(e0, st));
    tgk::mix_rate_kernel<tgk::kReadThreads><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
        static_cast<u64 *>(T.d), iters, 0x9E3779B97F4A7C15ull);
    TG_HIP(hipGetLastError());
    TG_HIP(hipEventRecord(e1, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    float ms = 0.f;
    TG_HIP(hipEventElapsedTime(&ms, e0, e1));
    if (!(ms > 0.f)) return TG_ERR_HIP;
    *words_per_s = double(grid) * tgk::kReadThreads * double(iters) * 16.0 / (double(ms) * 1e-3);
    return TG_OK;
}

tg_status tg_host_device_ptr(const void *pinned, void **out_dev) {
    if (!pinned || !out_dev) return TG_ERR_INVALID;
    void *dev = device_mapping(pinned);
    if (!dev) return TG_ERR_INVALID;
    *out_dev = dev;
    return TG_OK;
}

void tg_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_shared.mu);
    g_shared.t.shutdown();
}

const char *tg_strerror(tg_status s) {
    switch (s) {
        case TG_OK: return "ok";
        case TG_ERR_INVALID: return "invalid argument";
        case TG_ERR_NOSPACE: return "no space in pool";
        case TG_ERR_STALE: return "plan is stale";
        case TG_ERR_NOTFOUND: return "model not found";
        case TG_ERR_HIP: return "HIP call failed";
        case TG_ERR_NOMEM: return "out of memory";
        case TG_ERR_CORRUPT: return "assembled bytes do not match fingerprint";
        default: return "unknown status";
    }
}

}  // extern "C"
