// C ABI of the Load path (see include/tangram.h): argument checks, descriptor
// tables, kernel launches, the host-to-device side stream and commit.
#include "../../include/tangram.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hip.h"
#include "reuse_store.h"

struct tg_pool { tg::ReuseStore store; tg_pool(uint64_t b, uint64_t c, uint32_t a) : store(b, c, a) {} };
struct tg_load_plan { tg::Plan plan; std::vector<tg_plan_op> rows; std::vector<tg_move> move_rows; };

namespace {

using tgk::u32;
using tgk::u64;

#define TG_HIP(call) do { if ((call) != hipSuccess) { (void)hipGetLastError(); return TG_ERR_HIP; } } while (0)

// Loads in flight per lane (U) and resident workgroups per compute unit for
// each kernel.  Chosen by measurement on MI355X; see tg_set_tuning.
tg_tuning g_tune = {8, 4, 4, 1, 4, 2, uint64_t(64) << 10};

bool g_profiling = false;
tg_timing g_timing = {};

// A move whose source and destination overlap goes through this much staging at a time.
constexpr size_t kBounceBytes = size_t(128) << 20;
// A stretch of moves whose first byte shifts by at least this much is copied
// straight (up to that many bytes per launch); below it launches would be too
// small to be worth their launch cost and the stretch is staged.
constexpr uint64_t kDirectShift = uint64_t(32) << 20;

// A verifying tg_assemble cuts the host-to-device copies into this many batches
// and fingerprints each as soon as it has landed.
constexpr size_t kVerifyBatches = 4;
// ... but only batches of at least this many bytes: a dependency between two
// streams costs far more than a small copy (measured: a 9 MB model loads in
// 0.16 ms when the host joins the streams and in 1.4 ms with four event waits).
constexpr uint64_t kVerifyBatchMinBytes = uint64_t(64) << 20;
// Events: 0-1 gather, 2-3 host-to-device stream, 4-5 moves, 6.. one pair per
// verification group (gather, the batches, the moved tensors), then one per batch.
constexpr int kBatchEvent0 = 6 + 2 * int(2 + kVerifyBatches);
// ... and, for the second host-to-device stream, one more per batch and one for its end
constexpr int kBatch2Event0 = kBatchEvent0 + int(kVerifyBatches);
constexpr int kSecondDoneEvent = kBatch2Event0 + int(kVerifyBatches);
constexpr int kEvents = kSecondDoneEvent + 1;

// Library-owned scratch: one pinned staging buffer and one device buffer that
// hold a launch's descriptor table, tile prefix and result words.
struct Scratch {
    std::mutex mu;
    void *h = nullptr, *d = nullptr;
    size_t cap = 0;
    int cu_count = 0;
    int device = -1;                    // the one device this process's scratch lives on
    hipEvent_t ev[kEvents] = {};
    void *bounce = nullptr;             // staging for moves whose source and destination overlap

    tg_status init() {
        int dev = 0;
        TG_HIP(hipGetDevice(&dev));
        if (cu_count != 0) return dev == device ? TG_OK : TG_ERR_INVALID;
        hipDeviceProp_t prop;
        TG_HIP(hipGetDeviceProperties(&prop, dev));
        for (auto &e : ev)
            if (!e) TG_HIP(hipEventCreate(&e));
        cu_count = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        device = dev;
        return TG_OK;
    }
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
    void shutdown() {
        release_buffers();
        if (bounce) { (void)hipFree(bounce); bounce = nullptr; }
        for (auto &e : ev) if (e) { (void)hipEventDestroy(e); e = nullptr; }
        cu_count = 0;
        device = -1;
    }
} g_scratch;

size_t align_up(size_t n, size_t a) { return (n + a - 1) / a * a; }

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

u32 grid_for(u32 total_tiles, u32 wgs_per_cu) {
    const u64 resident = u64(g_scratch.cu_count) * std::max<u32>(1, wgs_per_cu);
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

// ---- fingerprint over device-visible spans; scratch lock held by the caller
tg_status fingerprint_locked(const tg_span *spans, u32 n, uint64_t *out_fp, hipStream_t st,
                             float *ms_out, uint64_t *bytes_out) {
    const u32 U = pick_u(g_tune.fingerprint_unroll);
    const TableLayout L = table_layout(n, sizeof(tgk::Span), sizeof(u64));
    tg_status rc = g_scratch.ensure(L.total);
    if (rc != TG_OK) return rc;
    char *h = static_cast<char *>(g_scratch.h), *d = static_cast<char *>(g_scratch.d);
    tgk::Span *hs = reinterpret_cast<tgk::Span *>(h + L.desc_off);
    u64 total_bytes = 0;
    for (u32 i = 0; i < n; ++i) {
        hs[i].ptr = u64(reinterpret_cast<uintptr_t>(spans[i].ptr));
        hs[i].nbytes = spans[i].nbytes;
        total_bytes += spans[i].nbytes;
    }
    u32 *hp = reinterpret_cast<u32 *>(h + L.prefix_off);
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Span) / 8, n, tile_for(tgk::kReadThreads, U))) return TG_ERR_INVALID;
    const u32 total_tiles = hp[n];
    u64 *d_out = reinterpret_cast<u64 *>(d + L.result_off);
    u64 *h_out = reinterpret_cast<u64 *>(h + L.result_off);
    DrainOnExit drain(st);
    TG_HIP(hipMemcpyAsync(d, h, L.result_off, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(tgk::zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, st, d_out, n);
    if (total_tiles > 0) {
        const u32 grid = grid_for(total_tiles, g_tune.fingerprint_wgs_per_cu);
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[0], st));
        const u32 run = run_for(total_tiles, grid);
        TG_FOR_U(U, tgk::fingerprint_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
                        reinterpret_cast<const tgk::Span *>(d + L.desc_off),
                        reinterpret_cast<const u32 *>(d + L.prefix_off), n, run, d_out));
        TG_HIP(hipGetLastError());
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[1], st));
    }
    TG_HIP(hipMemcpyAsync(h_out, d_out, n * sizeof(u64), hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    if (g_profiling && ms_out) {
        float ms = 0.f;
        if (total_tiles > 0) TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[0], g_scratch.ev[1]));
        *ms_out = ms;
        if (bytes_out) *bytes_out = total_bytes;
    }
    std::memcpy(out_fp, h_out, n * sizeof(u64));
    return TG_OK;
}

tg_status compare_locked(const tg_pair *pairs, u32 n, uint32_t *out_differs, hipStream_t st) {
    const u32 U = pick_u(g_tune.compare_unroll);
    const TableLayout L = table_layout(n, sizeof(tgk::Pair), sizeof(u64));
    tg_status rc = g_scratch.ensure(L.total);
    if (rc != TG_OK) return rc;
    char *h = static_cast<char *>(g_scratch.h), *d = static_cast<char *>(g_scratch.d);
    tgk::Pair *hs = reinterpret_cast<tgk::Pair *>(h + L.desc_off);
    u64 total_bytes = 0;
    for (u32 i = 0; i < n; ++i) {
        hs[i].a = u64(reinterpret_cast<uintptr_t>(pairs[i].a));
        hs[i].b = u64(reinterpret_cast<uintptr_t>(pairs[i].b));
        hs[i].nbytes = pairs[i].nbytes;
        total_bytes += pairs[i].nbytes;
    }
    u32 *hp = reinterpret_cast<u32 *>(h + L.prefix_off);
    if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Pair) / 8, n, tile_for(tgk::kReadThreads, U))) return TG_ERR_INVALID;
    const u32 total_tiles = hp[n];
    // results are 32-bit flags; the zero kernel clears whole 64-bit words
    u32 *d_out = reinterpret_cast<u32 *>(d + L.result_off);
    u32 *h_out = reinterpret_cast<u32 *>(h + L.result_off);
    DrainOnExit drain(st);
    TG_HIP(hipMemcpyAsync(d, h, L.result_off, hipMemcpyHostToDevice, st));
    const u32 words = (n + 1) / 2;
    hipLaunchKernelGGL(tgk::zero_words_kernel, dim3((words + 255) / 256), dim3(256), 0, st,
                       reinterpret_cast<u64 *>(d_out), words);
    if (total_tiles > 0) {
        const u32 grid = grid_for(total_tiles, g_tune.compare_wgs_per_cu);
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[0], st));
        const u32 run = run_for(total_tiles, grid);
        TG_FOR_U(U, tgk::compare_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, st>>>(
                        reinterpret_cast<const tgk::Pair *>(d + L.desc_off),
                        reinterpret_cast<const u32 *>(d + L.prefix_off), n, run, d_out));
        TG_HIP(hipGetLastError());
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[1], st));
    }
    TG_HIP(hipMemcpyAsync(h_out, d_out, n * sizeof(u32), hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    drain.armed = false;
    if (g_profiling) {
        float ms = 0.f;
        if (total_tiles > 0) TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[0], g_scratch.ev[1]));
        g_timing.compare_ms = ms;
        g_timing.compare_bytes = total_bytes;
    }
    std::memcpy(out_differs, h_out, n * sizeof(u32));
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
tg_status build_move_launches(const std::vector<tg::Move> &moves, uint64_t base,
                              std::vector<std::vector<tgk::Copy>> &launches, u64 &traffic) {
    traffic = 0;
    const u64 bounce = u64(reinterpret_cast<uintptr_t>(g_scratch.bounce));
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
                in.push_back(tgk::Copy{base + d, base + s, len});
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
                in.push_back(tgk::Copy{bounce + staged, base + s, len});
                out.push_back(tgk::Copy{base + d, bounce + staged, len});
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
        if (!out.empty()) launches.push_back(std::move(out));
    }
    return TG_OK;
}

// Inside one copy launch reads and writes are concurrent: no destination may
// touch a source of the same launch, and every extent lies in the pool or in
// the staging buffer.  A mistake in the cutting above then comes back as an
// error code instead of moved tensors that overwrote each other.
tg_status check_move_launches(const std::vector<std::vector<tgk::Copy>> &launches, uint64_t base, uint64_t cap) {
    const u64 bounce = u64(reinterpret_cast<uintptr_t>(g_scratch.bounce));
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
        } else if (op.src_off > pl.host_bytes || op.nbytes > pl.host_bytes - op.src_off) {
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
    tensors.resize(m->n_tensors);
    for (u32 k = 0; k < m->n_tensors; ++k) {
        const tg_tensor_desc &t = m->tensors[k];
        if (t.nbytes == 0) return TG_ERR_INVALID;
        if (t.src_off > m->host_bytes || t.nbytes > m->host_bytes - t.src_off) return TG_ERR_INVALID;
        tensors[k] = tg::TensorIn{t.nbytes, t.fp, t.src_off};
    }
    return TG_OK;
}

}  // namespace

extern "C" {

tg_status tg_pool_create(void *dev_base, uint64_t capacity, uint32_t align, tg_pool **out) {
    if (!dev_base || !out || capacity == 0) return TG_ERR_INVALID;
    if (align < 16 || (align & (align - 1)) != 0) return TG_ERR_INVALID;
    const uint64_t base = uint64_t(reinterpret_cast<uintptr_t>(dev_base));
    if (base % align != 0 || capacity % align != 0) return TG_ERR_INVALID;
    if (base + capacity < base) return TG_ERR_INVALID;
    tg_pool *p = new (std::nothrow) tg_pool(base, capacity, align);
    if (!p) return TG_ERR_NOMEM;
    *out = p;
    return TG_OK;
}

tg_status tg_pool_destroy(tg_pool *pool) {
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

tg_status tg_pool_entries(const tg_pool *pool, tg_entry *out, uint32_t cap, uint32_t *n) {
    if (!pool || !n || (cap > 0 && !out)) return TG_ERR_INVALID;
    const std::vector<const tg::Entry *> rows = pool->store.entries_by_offset();
    for (size_t i = 0; i < rows.size() && i < cap; ++i)
        out[i] = tg_entry{rows[i]->off, rows[i]->nbytes, rows[i]->fp, uint32_t(rows[i]->owners.size()),
                          rows[i]->active_refs};
    *n = uint32_t(rows.size());
    return TG_OK;
}

tg_status tg_fingerprint(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream) {
    if (n == 0) return TG_OK;
    if (!spans || !out_fp) return TG_ERR_INVALID;
    for (u32 i = 0; i < n; ++i) {
        if (spans[i].nbytes != 0 && !spans[i].ptr) return TG_ERR_INVALID;
        if (!aligned16(spans[i].ptr)) return TG_ERR_INVALID;
    }
    std::vector<uint64_t> tmp;
    try { tmp.resize(n); } catch (...) { return TG_ERR_NOMEM; }
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    const tg_status rc = fingerprint_locked(spans, n, tmp.data(), static_cast<hipStream_t>(stream),
                                            &g_timing.fingerprint_ms, &g_timing.fingerprint_bytes);
    if (rc == TG_OK) std::memcpy(out_fp, tmp.data(), n * sizeof(uint64_t));
    return rc;
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

tg_status tg_compare(const tg_pair *pairs, uint32_t n, uint32_t *out_differs, void *stream) {
    if (n == 0) return TG_OK;
    if (!pairs || !out_differs) return TG_ERR_INVALID;
    for (u32 i = 0; i < n; ++i) {
        if (pairs[i].nbytes != 0 && (!pairs[i].a || !pairs[i].b)) return TG_ERR_INVALID;
        if (!aligned16(pairs[i].a) || !aligned16(pairs[i].b)) return TG_ERR_INVALID;
    }
    std::vector<uint32_t> tmp;
    try { tmp.resize(n); } catch (...) { return TG_ERR_NOMEM; }
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    const tg_status rc = compare_locked(pairs, n, tmp.data(), static_cast<hipStream_t>(stream));
    if (rc == TG_OK) std::memcpy(out_differs, tmp.data(), n * sizeof(uint32_t));
    return rc;
}

tg_status tg_plan(tg_pool *pool, const tg_model_desc *model, uint32_t flags, void *stream,
                  tg_load_plan **out) {
    if (!pool || !out) return TG_ERR_INVALID;
    if (flags & ~(TG_PLAN_CONFIRM | TG_PLAN_EVICT | TG_PLAN_MERGE | TG_PLAN_ALIAS | TG_PLAN_PACK_TEXT))
        return TG_ERR_INVALID;
    const auto t0 = std::chrono::steady_clock::now();
    std::vector<tg::TensorIn> tensors;
    tg_status rc = check_model(model, tensors);
    if (rc != TG_OK) return rc;
    tg::ReuseStore &store = pool->store;
    if (store.model_active(model->model_id)) return TG_ERR_INVALID;
    const bool confirm = (flags & TG_PLAN_CONFIRM) != 0;
    if (confirm && !model->host_base) return TG_ERR_INVALID;

    const size_t n = tensors.size();
    std::vector<uint64_t> hits(n, 0);
    std::vector<std::pair<uint64_t, uint64_t>> cand;      // (offset, entry id), ascending offset
    if (!confirm) {
        // Section 3.1: a tensor found in the Tensor Mapping is reused.
        for (size_t k = 0; k < n; ++k) {
            store.candidates(tensors[k].fp, tensors[k].nbytes, cand);
            if (!cand.empty()) hits[k] = cand.front().second;
        }
    } else {
        // Every candidate of every tensor is compared with the incoming bytes
        // in one launch; the first candidate (lowest offset) that is equal wins.
        void *host_dev = nullptr;
        if (hipHostGetDevicePointer(&host_dev, const_cast<void *>(model->host_base), 0) != hipSuccess) {
            (void)hipGetLastError();
            return TG_ERR_INVALID;
        }
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
            }
        }
        if (!pairs.empty()) {
            std::vector<uint32_t> differs(pairs.size());
            std::lock_guard<std::mutex> lock(g_scratch.mu);
            rc = compare_locked(pairs.data(), u32(pairs.size()), differs.data(), static_cast<hipStream_t>(stream));
            if (rc != TG_OK) return rc;
            for (size_t i = 0; i < pairs.size(); ++i)
                if (!differs[i] && hits[who[i].first] == 0) hits[who[i].first] = who[i].second;
        }
    }

    tg_load_plan *lp = new (std::nothrow) tg_load_plan();
    if (!lp) return TG_ERR_NOMEM;
    lp->plan.model_id = model->model_id;
    lp->plan.host_base = model->host_base;
    lp->plan.host_bytes = model->host_bytes;
    const tg::Status ps = store.plan(tensors, hits, flags, lp->plan);
    if (ps != tg::OK) { delete lp; return tg_status(ps); }
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
    *out = lp;
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    if (g_profiling)
        g_timing.plan_host_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
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

void tg_plan_free(tg_load_plan *plan) { delete plan; }

tg_status tg_commit(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs) {
    if (!pool || !plan) return TG_ERR_INVALID;
    std::vector<uint64_t> dst;
    const tg::Status s = pool->store.commit(plan->plan, dst);
    if (s != tg::OK) return tg_status(s);
    if (out_dev_ptrs)
        for (size_t k = 0; k < dst.size(); ++k)
            out_dev_ptrs[k] = reinterpret_cast<void *>(uintptr_t(pool->store.base() + dst[k]));
    return TG_OK;
}

tg_status tg_abandon(tg_pool *pool, tg_load_plan *plan) {
    if (!pool || !plan) return TG_ERR_INVALID;
    return tg_status(pool->store.abandon(plan->plan));
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

tg_status tg_assemble_ex(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args, void **out_dev_ptrs) {
    if (!pool || !plan || !args) return TG_ERR_INVALID;
    if (args->flags & ~TG_ASSEMBLE_VERIFY) return TG_ERR_INVALID;
    const uint32_t flags = args->flags;
    void *stream_gather = args->stream_gather, *stream_h2d = args->stream_h2d;
    tg::ReuseStore &store = pool->store;
    tg::Plan &pl = plan->plan;
    if (pl.consumed || pl.pool_tag != &store) return TG_ERR_INVALID;
    if (pl.generation != store.generation()) return TG_ERR_STALE;
    if (store.model_active(pl.model_id)) return TG_ERR_INVALID;
    if (pl.transfer_bytes > 0 && !pl.host_base) return TG_ERR_INVALID;
    hipStream_t sg = static_cast<hipStream_t>(stream_gather), sh = static_cast<hipStream_t>(stream_h2d);
    // The copies may be dealt over two streams: one copy then starts while the other is still
    // running, which hides what a copy costs to start (about 10 us each on one stream).
    hipStream_t sh2 = args->use_second_h2d_stream ? static_cast<hipStream_t>(args->stream_h2d_second) : sh;
    const bool dual = sh2 != sh && sh2 != sg && sh != sg;
    if (!dual) sh2 = sh;
    const uint64_t base = store.base();
    {
        const tg_status rc = validate_plan(pl, store);
        if (rc != TG_OK) return rc;
    }

    std::lock_guard<std::mutex> lock(g_scratch.mu);
    {
        const tg_status rc = g_scratch.init();
        if (rc != TG_OK) return rc;
    }

    // ---- merge moves (Section 3.2, Stage 2), cut into launches whose reads and
    // writes do not meet
    std::vector<std::vector<tgk::Copy>> launches;
    u64 move_traffic = 0;
    if (!pl.moves.empty()) {
        tg_status rc = g_scratch.ensure_bounce();
        if (rc != TG_OK) return rc;
        rc = build_move_launches(pl.moves, base, launches, move_traffic);
        if (rc != TG_OK) return rc;
        rc = check_move_launches(launches, base, store.capacity());
        if (rc != TG_OK) return rc;
    }
    const size_t n_move_launches = launches.size();

    // Host-to-device list, in destination order; copies adjacent on both sides
    // (the slot padding included) are merged into one (Section 4 groups
    // adjacent tensors into large copies).
    struct H2D { uint64_t dst, src, len, padded; std::vector<u32> ops; };
    std::vector<H2D> h2d;
    std::vector<tgk::Copy> copies;
    const bool verify = (flags & TG_ASSEMBLE_VERIFY) != 0;
    // Verification groups: spans to fingerprint once the bytes are in place.
    // Group 0 holds what the gather launch writes (and aliased hits, already
    // in place); the host-to-device copies are cut into a few batches, each
    // verified on stream A as soon as its copies are done on stream B, so only
    // the last batch's fingerprint is left when the transfer ends.
    // A last group, if the plan moves resident tensors, holds those at their new
    // addresses (`moved`: its rows are pl.moves, not pl.ops).
    struct FpGroup {
        std::vector<u32> ops;
        bool moved = false;
        size_t desc_off = 0, prefix_off = 0, result_off = 0;
        u32 tiles = 0;
        u64 bytes = 0;
    };
    std::vector<FpGroup> groups(1);
    void *host_dev = nullptr;
    const uint64_t small = g_tune.h2d_kernel_max_bytes;
    if (small > 0 && pl.host_base &&
        hipHostGetDevicePointer(&host_dev, const_cast<void *>(pl.host_base), 0) != hipSuccess) {
        (void)hipGetLastError();
        host_dev = nullptr;
    }
    for (size_t k = 0; k < pl.ops.size(); ++k) {
        const tg::Op &op = pl.ops[k];
        if (op.kind == 0) {
            groups[0].ops.push_back(u32(k));
            if (pl.alias) continue;                      // used where it lies: nothing to copy
            copies.push_back(tgk::Copy{base + op.dst_off, base + op.src_off, op.nbytes});
        } else if (host_dev && op.nbytes <= small &&
                   ((uintptr_t(host_dev) + op.src_off) & 15u) == 0) {
            // small missing tensors ride in the gather launch, read through the
            // pinned buffer's device mapping, instead of one DMA call each
            groups[0].ops.push_back(u32(k));
            copies.push_back(tgk::Copy{base + op.dst_off, u64(uintptr_t(host_dev)) + op.src_off, op.nbytes});
        } else {
            h2d.push_back(H2D{op.dst_off, op.src_off, op.nbytes, store.round_up(op.nbytes), {u32(k)}});
        }
    }
    std::sort(h2d.begin(), h2d.end(), [](const H2D &a, const H2D &b) { return a.dst < b.dst; });
    std::vector<H2D> merged;
    u64 h2d_total = 0;
    for (const H2D &c : h2d) {
        h2d_total += c.len;
        if (!merged.empty()) {
            H2D &m = merged.back();
            if (m.dst + m.padded == c.dst && m.src + m.padded == c.src) {
                m.len = m.padded + c.len;
                m.padded += c.padded;
                m.ops.push_back(c.ops[0]);
                continue;
            }
        }
        merged.push_back(c);
    }
    // batch_end[j] = index one past the last merged copy of batch j
    std::vector<size_t> batch_end;
    if (!merged.empty()) {
        const size_t nb = !verify ? 1 : std::max<size_t>(1, std::min<size_t>(
            std::min<size_t>(kVerifyBatches, merged.size()), size_t(h2d_total / kVerifyBatchMinBytes)));
        // shares nb : nb-1 : ... : 1, so that little is left to fingerprint when the last copy lands
        const u64 denom = u64(nb) * (nb + 1) / 2;
        u64 acc = 0, cum = nb;
        for (size_t i = 0; i < merged.size(); ++i) {
            acc += merged[i].len;
            const size_t done = batch_end.size();
            if (i + 1 == merged.size() || (done + 1 < nb && acc * denom >= h2d_total * cum)) {
                batch_end.push_back(i + 1);
                cum += nb - (done + 1);
            }
        }
        if (verify) {
            size_t from = 0;
            for (size_t e : batch_end) {
                FpGroup g;
                for (size_t i = from; i < e; ++i) g.ops.insert(g.ops.end(), merged[i].ops.begin(), merged[i].ops.end());
                groups.push_back(std::move(g));
                from = e;
            }
        }
    }
    const size_t moved_group = groups.size();           // index of the moved tensors' group, if there is one
    if (verify && !pl.moves.empty()) {
        FpGroup g;
        g.moved = true;
        groups.push_back(std::move(g));
    }
    auto rows_of = [&](const FpGroup &g) { return g.moved ? pl.moves.size() : g.ops.size(); };
    u64 gather_bytes = 0;
    for (const auto &c : copies) gather_bytes += c.nbytes;
    if (!copies.empty()) launches.push_back(copies);

    // ---- one table upload for every launch of this call
    const u32 U = pick_u(g_tune.gather_unroll);
    const u64 tile = tile_for(tgk::kCopyThreads, U);
    const u32 FU = pick_u(g_tune.fingerprint_unroll);
    const u64 fp_tile = tile_for(tgk::kReadThreads, FU);
    struct Placed { size_t desc_off, prefix_off, ticket_off; u32 n, tiles; };
    std::vector<Placed> placed(launches.size());
    size_t table_bytes = 0;
    for (size_t i = 0; i < launches.size(); ++i) {
        const TableLayout L = table_layout(launches[i].size(), sizeof(tgk::Copy), 0);
        placed[i].desc_off = table_bytes + L.desc_off;
        placed[i].prefix_off = table_bytes + L.prefix_off;
        placed[i].ticket_off = table_bytes + L.total;    // the launch's tile counter, uploaded as zero
        placed[i].n = u32(launches[i].size());
        table_bytes += L.total + 256;
    }
    size_t results_off = 0, results_words = 0;
    if (verify) {
        for (FpGroup &g : groups) {
            const TableLayout L = table_layout(rows_of(g), sizeof(tgk::Span), 0);
            g.desc_off = table_bytes + L.desc_off;
            g.prefix_off = table_bytes + L.prefix_off;
            table_bytes += L.total;
        }
        results_off = table_bytes;                       // one result word per tensor, group after group
        for (FpGroup &g : groups) {
            g.result_off = results_off + results_words * sizeof(u64);
            results_words += rows_of(g);
        }
        table_bytes += align_up(results_words * sizeof(u64), 256);
    }
    DrainOnExit drain_gather(sg);
    drain_gather.armed = false;                 // nothing enqueued yet
    if (table_bytes > 0) {
        tg_status rc = g_scratch.ensure(table_bytes);
        if (rc != TG_OK) return rc;
        char *h = static_cast<char *>(g_scratch.h);
        for (size_t i = 0; i < launches.size(); ++i) {
            std::memcpy(h + placed[i].desc_off, launches[i].data(), launches[i].size() * sizeof(tgk::Copy));
            u32 *hp = reinterpret_cast<u32 *>(h + placed[i].prefix_off);
            if (!fill_prefix(hp, &launches[i][0].nbytes, sizeof(tgk::Copy) / 8, launches[i].size(), tile))
                return TG_ERR_INVALID;
            placed[i].tiles = hp[launches[i].size()];
            std::memset(h + placed[i].ticket_off, 0, 256);
        }
        if (verify) {
            for (FpGroup &g : groups) {
                const size_t rows = rows_of(g);
                if (rows == 0) continue;
                tgk::Span *hs = reinterpret_cast<tgk::Span *>(h + g.desc_off);
                for (size_t i = 0; i < rows; ++i) {
                    hs[i].ptr = base + (g.moved ? pl.moves[i].new_off : pl.ops[g.ops[i]].dst_off);
                    hs[i].nbytes = g.moved ? pl.moves[i].nbytes : pl.ops[g.ops[i]].nbytes;
                    g.bytes += hs[i].nbytes;
                }
                u32 *hp = reinterpret_cast<u32 *>(h + g.prefix_off);
                if (!fill_prefix(hp, &hs[0].nbytes, sizeof(tgk::Span) / 8, rows, fp_tile)) return TG_ERR_INVALID;
                g.tiles = hp[rows];
            }
        }
        TG_HIP(hipMemcpyAsync(g_scratch.d, g_scratch.h, verify ? results_off : table_bytes,
                              hipMemcpyHostToDevice, sg));
        drain_gather.armed = true;
        if (verify && results_words > 0) {
            tgk::zero_words_kernel<<<dim3(u32((results_words + 255) / 256)), dim3(256), 0, sg>>>(
                reinterpret_cast<u64 *>(static_cast<char *>(g_scratch.d) + results_off), u32(results_words));
            TG_HIP(hipGetLastError());
        }
    }
    auto launch_copy = [&](size_t i) -> tg_status {
        if (placed[i].tiles == 0) return TG_OK;
        char *d = static_cast<char *>(g_scratch.d);
        const u32 grid = grid_for(placed[i].tiles, g_tune.gather_wgs_per_cu);
        TG_FOR_U(U, tgk::gather_kernel<tgk::kCopyThreads, kU><<<dim3(grid), dim3(tgk::kCopyThreads), 0, sg>>>(
                        reinterpret_cast<const tgk::Copy *>(d + placed[i].desc_off),
                        reinterpret_cast<const u32 *>(d + placed[i].prefix_off), placed[i].n,
                        reinterpret_cast<u32 *>(d + placed[i].ticket_off)));
        TG_HIP(hipGetLastError());
        return TG_OK;
    };
    // fingerprint of verification group gi on stream A (events 6+2gi, 7+2gi time it)
    auto launch_verify = [&](size_t gi) -> tg_status {
        const FpGroup &g = groups[gi];
        if (g.tiles == 0) return TG_OK;
        char *d = static_cast<char *>(g_scratch.d);
        const u32 grid = grid_for(g.tiles, g_tune.fingerprint_wgs_per_cu);
        const u32 run = run_for(g.tiles, grid);
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[6 + 2 * gi], sg));
        TG_FOR_U(FU, tgk::fingerprint_kernel<tgk::kReadThreads, kU><<<dim3(grid), dim3(tgk::kReadThreads), 0, sg>>>(
                         reinterpret_cast<const tgk::Span *>(d + g.desc_off),
                         reinterpret_cast<const u32 *>(d + g.prefix_off), u32(rows_of(g)), run,
                         reinterpret_cast<u64 *>(d + g.result_off)));
        TG_HIP(hipGetLastError());
        if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[7 + 2 * gi], sg));
        return TG_OK;
    };

    // Everything that touches the pool's bytes: once this has started, a
    // failure may leave some of the plan's writes done.
    std::vector<uint64_t> corrupt_moved;                  // moved tensors that no longer match their rows
    auto device_work = [&]() -> tg_status {
        // ---- moves first (stream A); nothing may land in the pool before they are done
        if (n_move_launches > 0) {
            if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[4], sg));
            for (size_t i = 0; i < n_move_launches; ++i) {
                const tg_status rc = launch_copy(i);
                if (rc != TG_OK) return rc;
            }
            TG_HIP(hipEventRecord(g_scratch.ev[5], sg));
            if (sh != sg) TG_HIP(hipStreamWaitEvent(sh, g_scratch.ev[5], 0));
            if (dual) TG_HIP(hipStreamWaitEvent(sh2, g_scratch.ev[5], 0));
            if (verify) {                                 // the moved tensors, where they are now
                const tg_status rc = launch_verify(moved_group);
                if (rc != TG_OK) return rc;
            }
        }

        // ---- gather launch (stream A), then the fingerprint of what it wrote
        if (!copies.empty()) {
            if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[0], sg));
            const tg_status rc = launch_copy(launches.size() - 1);
            if (rc != TG_OK) return rc;
            if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[1], sg));
        }
        if (verify) {
            const tg_status rc = launch_verify(0);
            if (rc != TG_OK) return rc;
        }

        // ---- host-to-device copies (stream B), overlapped with the gather; each
        // batch is fingerprinted on stream A as soon as it has landed
        u64 h2d_bytes = 0;
        if (!merged.empty()) {
            if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[2], sh));
            size_t from = 0;
            for (size_t j = 0; j < batch_end.size(); ++j) {
                bool used2 = false;
                for (size_t i = from; i < batch_end[j]; ++i) {
                    const H2D &c = merged[i];
                    const bool second = dual && (i & 1) != 0;
                    TG_HIP(hipMemcpyAsync(reinterpret_cast<void *>(uintptr_t(base + c.dst)),
                                          static_cast<const char *>(pl.host_base) + c.src, c.len,
                                          hipMemcpyHostToDevice, second ? sh2 : sh));
                    used2 = used2 || second;
                    h2d_bytes += c.len;
                }
                from = batch_end[j];
                if (verify) {
                    if (sh != sg && h2d_total < kVerifyBatchMinBytes) {
                        TG_HIP(hipStreamSynchronize(sh));        // small transfer: the host joins
                        if (used2) TG_HIP(hipStreamSynchronize(sh2));
                    } else if (sh != sg) {
                        TG_HIP(hipEventRecord(g_scratch.ev[kBatchEvent0 + j], sh));
                        TG_HIP(hipStreamWaitEvent(sg, g_scratch.ev[kBatchEvent0 + j], 0));
                        if (used2) {
                            TG_HIP(hipEventRecord(g_scratch.ev[kBatch2Event0 + j], sh2));
                            TG_HIP(hipStreamWaitEvent(sg, g_scratch.ev[kBatch2Event0 + j], 0));
                        }
                    }
                    const tg_status rc = launch_verify(1 + j);
                    if (rc != TG_OK) return rc;
                }
            }
            if (dual) {                                   // stream B's end event covers the second stream
                TG_HIP(hipEventRecord(g_scratch.ev[kSecondDoneEvent], sh2));
                TG_HIP(hipStreamWaitEvent(sh, g_scratch.ev[kSecondDoneEvent], 0));
            }
            if (g_profiling) TG_HIP(hipEventRecord(g_scratch.ev[3], sh));
        }
        if (verify && results_words > 0)
            TG_HIP(hipMemcpyAsync(static_cast<char *>(g_scratch.h) + results_off,
                                  static_cast<char *>(g_scratch.d) + results_off, results_words * sizeof(u64),
                                  hipMemcpyDeviceToHost, sg));

        // ---- join
        TG_HIP(hipStreamSynchronize(sg));
        if (sh != sg) TG_HIP(hipStreamSynchronize(sh));
        if (dual) TG_HIP(hipStreamSynchronize(sh2));
        if (g_profiling) {
            float ms = 0.f;
            if (!copies.empty()) TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[0], g_scratch.ev[1]));
            g_timing.gather_ms = ms;
            g_timing.gather_bytes = gather_bytes;
            ms = 0.f;
            if (!merged.empty()) TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[2], g_scratch.ev[3]));
            g_timing.h2d_ms = ms;
            g_timing.h2d_bytes = h2d_bytes;
            g_timing.h2d_copies = u32(merged.size());
            ms = 0.f;
            if (n_move_launches > 0) TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[4], g_scratch.ev[5]));
            g_timing.move_ms = ms;
            g_timing.move_bytes = pl.moved_bytes;
            g_timing.move_traffic_bytes = move_traffic;
            g_timing.move_launches = u32(n_move_launches);
            if (verify) {
                float total = 0.f;
                u64 bytes = 0;
                u32 launched = 0;
                for (size_t gi = 0; gi < groups.size(); ++gi) {
                    if (groups[gi].tiles == 0) continue;
                    TG_HIP(hipEventElapsedTime(&ms, g_scratch.ev[6 + 2 * gi], g_scratch.ev[7 + 2 * gi]));
                    total += ms;
                    bytes += groups[gi].bytes;
                    ++launched;
                }
                g_timing.verify_ms = total;
                g_timing.verify_bytes = bytes;
                g_timing.verify_launches = launched;
            }
        }

        // ---- the integrity check proper: every slot's fingerprint against its descriptor,
        // every moved tensor's against its row of the Tensor Mapping
        if (verify) {
            const u64 *res = reinterpret_cast<const u64 *>(static_cast<char *>(g_scratch.h) + results_off);
            size_t at = 0;
            bool good = true;
            for (const FpGroup &g : groups) {
                if (g.moved) {
                    for (const tg::Move &m : pl.moves)
                        if (res[at++] != m.fp) { corrupt_moved.push_back(m.entry); good = false; }
                } else {
                    for (u32 k : g.ops)
                        if (res[at++] != pl.fps[k]) good = false;
                }
            }
            if (!good) return TG_ERR_CORRUPT;
        }
        return TG_OK;
    };
    {
        const tg_status rc = device_work();
        if (rc != TG_OK) {
            // nothing of this call may still be running when the tables are reused
            (void)hipStreamSynchronize(sg);
            if (sh != sg) (void)hipStreamSynchronize(sh);
            if (dual) (void)hipStreamSynchronize(sh2);
            (void)hipGetLastError();
            // evicted tensors may have been overwritten and moved ones have moved:
            // record that much, so that the mapping describes the pool's bytes
            if (!pl.moves.empty() || !pl.evict.empty()) (void)store.abandon(pl);
            store.drop_corrupt(corrupt_moved);
            return rc;
        }
    }

    drain_gather.armed = false;                 // both streams have been waited for

    // ---- commit (Section 3.1: update the mapping, return the addresses)
    std::vector<uint64_t> dst;
    const tg::Status s = store.commit(pl, dst);
    if (s != tg::OK) return tg_status(s);
    if (out_dev_ptrs)
        for (size_t k = 0; k < dst.size(); ++k)
            out_dev_ptrs[k] = reinterpret_cast<void *>(uintptr_t(base + dst[k]));
    return TG_OK;
}

tg_status tg_release(tg_pool *pool, uint64_t model_id, uint32_t flags) {
    if (!pool) return TG_ERR_INVALID;
    return tg_status(pool->store.release(model_id, (flags & TG_RELEASE_EVICT) != 0));
}

tg_status tg_set_model_cost(tg_pool *pool, uint64_t model_id, double miss_prob, double load_bw, double alpha) {
    if (!pool) return TG_ERR_INVALID;
    return tg_status(pool->store.set_model_cost(model_id, miss_prob, load_bw, alpha));
}

tg_status tg_reuse_size(const tg_pool *pool, const tg_model_desc *model, double link_bytes_per_s,
                        uint64_t *reuse_bytes, double *est_load_s) {
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
}

void tg_set_profiling(int on) {
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    g_profiling = on != 0;
    g_timing = tg_timing{};
}

tg_status tg_last_timing(tg_timing *out) {
    if (!out) return TG_ERR_INVALID;
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    *out = g_timing;
    return TG_OK;
}

tg_status tg_set_tuning(const tg_tuning *t) {
    if (!t) return TG_ERR_INVALID;
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    g_tune = *t;
    return TG_OK;
}

tg_status tg_get_tuning(tg_tuning *t) {
    if (!t) return TG_ERR_INVALID;
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    *t = g_tune;
    return TG_OK;
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

void tg_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    g_scratch.shutdown();
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
