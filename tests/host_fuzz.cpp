// Random histories against the host-side Reuse Store, built with
// -fsanitize=address,undefined and with -fsanitize=thread by
// tests/test_host_sanitizers.py.  Checks the structural invariants after every
// step; the sanitizers check the rest.  With a second argument the histories
// are dealt over that many threads, each with stores of its own: the stores
// share nothing, which is what ThreadSanitizer then confirms.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <thread>
#include <vector>

#include "../paper_2512_01357_amd/csrc/reuse_store.h"

using namespace tg;

static void fail(const char *what, int step) {
    std::fprintf(stderr, "invariant broken at step %d: %s\n", step, what);
    std::exit(1);
}

static void run_history(unsigned seed) {
    {
        std::mt19937_64 rng(seed);
        const uint64_t cap = 256ull * (64 + rng() % 400);
        ReuseStore store(1ull << 40, cap, 256);
        const uint64_t sizes[] = {40, 256, 300, 512, 1000, 1024, 2048, 3000, 6000};
        std::vector<uint64_t> running, retained;
        uint64_t next_id = 1;
        for (int step = 0; step < 400; ++step) {
            const double r = double(rng() % 1000) / 1000.0;
            if (r < 0.5 || (running.empty() && retained.empty())) {
                const size_t n = 1 + rng() % 7;
                std::vector<TensorIn> tensors(n);
                uint64_t at = 0;
                for (auto &t : tensors) {
                    const uint64_t content = rng() % 30;
                    t.nbytes = sizes[content % 9];
                    t.fp = content * 0x9E3779B97F4A7C15ull + 12345;
                    t.src_off = at;
                    at += (t.nbytes + 255) / 256 * 256;
                }
                uint64_t mid = next_id;
                if (!retained.empty() && rng() % 4 == 0) mid = retained[rng() % retained.size()];
                if (rng() % 3 == 0) store.set_model_cost(mid, 0.1 + double(rng() % 10) / 10.0, 1.0 + double(rng() % 5), 1.0);
                uint32_t flags = 0;
                if (rng() % 10 < 7) flags |= PLAN_EVICT;
                if (rng() % 10 < 7) flags |= PLAN_MERGE;
                if (rng() % 2) flags |= PLAN_ALIAS;
                if (rng() % 2) flags |= PLAN_PACK_TEXT;
                if (rng() % 3 == 0) flags |= PLAN_CAP_TEXT;
                std::vector<uint64_t> hits(n, 0);
                std::vector<std::pair<uint64_t, uint64_t>> cand;
                for (size_t k = 0; k < n; ++k) {
                    store.candidates(tensors[k].fp, tensors[k].nbytes, cand);
                    if (!cand.empty()) hits[k] = cand.front().second;
                }
                Plan plan;
                plan.model_id = mid;
                const Stats before = store.stats();
                const Status ps = store.plan(tensors, hits, flags, plan);
                const Stats after_plan = store.stats();
                if (before.free_bytes != after_plan.free_bytes || before.n_entries != after_plan.n_entries ||
                    before.n_regions != after_plan.n_regions)
                    fail("planning changed the pool", step);
                if (ps == ERR_NOSPACE) continue;
                if (ps != OK) fail("unexpected plan status", step);
                // destinations of new slots and moved tensors are pairwise disjoint
                std::vector<std::pair<uint64_t, uint64_t>> ext;
                for (size_t k = 0; k < n; ++k)
                    if (!(plan.alias && hits[k] != 0)) ext.push_back({plan.ops[k].dst_off, plan.ops[k].dst_off + plan.ops[k].nbytes});
                for (const Move &m : plan.moves) {
                    if (m.new_off >= m.old_off) fail("a move does not go down", step);
                    ext.push_back({m.new_off, m.new_off + m.nbytes});
                }
                std::sort(ext.begin(), ext.end());
                for (size_t i = 1; i < ext.size(); ++i)
                    if (ext[i].first < ext[i - 1].second) fail("overlapping destinations", step);
                if (plan.moved_bytes > plan.merge_bound && !plan.moves.empty()) fail("moved more than the bound", step);
                std::vector<uint64_t> dst;
                if (rng() % 10 == 0) continue;            // planned, never carried out
                if (rng() % 12 == 0) {                    // given up half way
                    const uint64_t free_before = store.stats().free_bytes;
                    if (store.abandon(plan) != OK) fail("abandon failed", step);
                    if (store.abandon(plan) != ERR_INVALID) fail("a plan was abandoned twice", step);
                    if (store.stats().free_bytes != free_before + plan.evicted_bytes) fail("abandon: free bytes", step);
                    continue;
                }
                if (store.commit(plan, dst) != OK) fail("commit failed", step);
                if (store.commit(plan, dst) != ERR_INVALID) fail("a plan was committed twice", step);
                running.push_back(mid);
                for (size_t i = 0; i < retained.size(); ++i)
                    if (retained[i] == mid) { retained.erase(retained.begin() + i); break; }
                if (mid == next_id) ++next_id;
            } else if (!running.empty() && (retained.empty() || rng() % 10 < 6)) {
                const size_t i = rng() % running.size();
                const bool evict = rng() % 10 < 4;
                if (store.release(running[i], evict) != OK) fail("release of a running model failed", step);
                if (!evict) retained.push_back(running[i]);
                running.erase(running.begin() + i);
            } else {
                const size_t i = rng() % retained.size();
                const Status s = store.release(retained[i], true);
                if (s != OK && s != ERR_NOTFOUND) fail("release of a retained model failed", step);
                retained.erase(retained.begin() + i);
            }
            if (rng() % 40 == 0) {                        // a resident tensor turns out to be damaged
                const auto rows = store.entries_by_offset();
                if (!rows.empty()) {
                    const Entry *e = rows[rng() % rows.size()];
                    const bool in_use = e->active_refs != 0;
                    const Stats b = store.stats();
                    const uint64_t slot = store.round_up(e->nbytes);
                    store.drop_corrupt({e->id});
                    const Stats a = store.stats();
                    if (in_use ? (a.n_entries != b.n_entries || a.free_bytes != b.free_bytes)
                               : (a.n_entries + 1 != b.n_entries || a.free_bytes != b.free_bytes + slot))
                        fail("drop_corrupt", step);
                    // models that lost their last retained tensor are gone
                    std::vector<uint64_t> still;
                    for (uint64_t m : retained)
                        if (store.release(m, false) == OK) still.push_back(m);
                    retained.swap(still);
                }
            }
            const Stats st = store.stats();
            if (st.free_bytes > st.capacity || st.largest_free > st.free_bytes) fail("free bytes", step);
            if (st.n_regions < st.n_free_regions + st.n_entries) fail("region count", step);
            if (st.n_active > st.n_entries) fail("active count", step);
        }
    }
}

int main(int argc, char **argv) {
    const unsigned seeds = argc > 1 ? unsigned(std::atoi(argv[1])) : 20;
    const unsigned n_threads = argc > 2 ? unsigned(std::atoi(argv[2])) : 1;
    if (n_threads <= 1) {
        for (unsigned seed = 0; seed < seeds; ++seed) run_history(seed);
    } else {
        std::vector<std::thread> threads;
        for (unsigned t = 0; t < n_threads; ++t)
            threads.emplace_back([=] { for (unsigned seed = t; seed < seeds; seed += n_threads) run_history(seed); });
        for (auto &th : threads) th.join();
    }
    std::printf("ok %u histories\n", seeds);
    return 0;
}
