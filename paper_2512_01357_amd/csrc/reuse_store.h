// Host-side Reuse Store: Region List, Tensor Mapping and the load planner.
//
// Pure C++ (no HIP): everything here runs on the CPU and decides *what* the
// device will be asked to do.  Follows the paper's Section 3.1 (Tensor
// Mapping lookup, return addresses), Section 3.2 (regions in physical order,
// best-fit allocation, Stage 1 minimal-cost eviction with Eq. 2, Stage 2
// Partitioned-Gain Packing, Algorithm 1) and Eq. 3.
#pragma once

#include <cstddef>
#include <cstdint>
#include <map>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

namespace tg {

enum Status : int32_t {
    OK = 0, ERR_INVALID = -1, ERR_NOSPACE = -2, ERR_STALE = -3, ERR_NOTFOUND = -4, ERR_HIP = -5,
    ERR_NOMEM = -6, ERR_CORRUPT = -7
};

enum PlanFlags : uint32_t {
    PLAN_CONFIRM = 1, PLAN_EVICT = 2, PLAN_MERGE = 4, PLAN_ALIAS = 8, PLAN_PACK_TEXT = 16, PLAN_CAP_TEXT = 32
};

// Region tags: 0 = none, otherwise an entry id; ids at or above kNewTag mark
// the slot of tensor (tag - kNewTag) of a plan that has not been committed.
constexpr uint64_t kNewTag = uint64_t(1) << 62;

struct Entry {                       // one row of the Tensor Mapping
    uint64_t id = 0;
    uint64_t off = 0;                // slot offset in the pool
    uint64_t nbytes = 0;             // tensor length (slot is roundup(nbytes, align))
    uint64_t fp = 0;
    uint32_t active_refs = 0;        // running models that use it
    std::vector<uint64_t> owners;    // models that list it, oldest first
};

struct Key {
    uint64_t fp, nbytes;
    bool operator==(const Key &o) const { return fp == o.fp && nbytes == o.nbytes; }
};
struct KeyHash {
    size_t operator()(const Key &k) const {
        // fp is already well mixed; fold the length in so equal contents of
        // different lengths land in different buckets
        return static_cast<size_t>(k.fp ^ (k.nbytes * 0x9E3779B97F4A7C15ull));
    }
};

struct Region { uint64_t len; bool free; uint64_t tag; };

// Section 3.2: regions chained in physical order, each free or allocated,
// plus an index of the free ones by (length, offset) so that best fit is one
// lower_bound.
class RegionList {
public:
    RegionList() = default;
    explicit RegionList(uint64_t capacity);

    bool best_fit(uint64_t need, uint64_t &off) const;     // smallest free region >= need, lowest offset
    void take(uint64_t off, uint64_t need, uint64_t tag);   // carve the low end of the free region at off
    void give(uint64_t off);                                // free the region at off, merge neighbours
    void set_tag(uint64_t off, uint64_t tag) { by_off_.at(off).tag = tag; }

    uint64_t free_bytes() const { return free_bytes_; }
    uint64_t largest_free() const { return free_idx_.empty() ? 0 : free_idx_.rbegin()->first; }
    size_t size() const { return by_off_.size(); }
    size_t n_free() const { return free_idx_.size(); }
    const std::map<uint64_t, Region> &regions() const { return by_off_; }

    struct Flat { uint64_t off, len; bool free; uint64_t tag; };
    std::vector<Flat> flatten() const;
    void splice(uint64_t start, uint64_t end, const std::vector<Flat> &flats);

private:
    std::map<uint64_t, Region> by_off_;
    std::set<std::pair<uint64_t, uint64_t>> free_idx_;      // (len, off)
    uint64_t free_bytes_ = 0;
};

struct TensorIn {         // one incoming tensor
    uint64_t nbytes, fp, src_off;
};

struct Op {               // decision for one incoming tensor
    uint32_t kind;        // 0 reuse, 1 host-to-device
    uint64_t dst_off, src_off, nbytes;
};

struct Move { uint64_t entry, old_off, new_off, nbytes, fp; };

struct Plan {
    uint64_t              model_id = 0;
    const void           *host_base = nullptr;
    uint64_t              host_bytes = 0;
    uint64_t              generation = 0;
    const void           *pool_tag = nullptr;   // the store the plan was made for
    bool                  alias = false;
    std::vector<Op>       ops;                  // model order
    std::vector<uint64_t> fps;                  // model order
    std::vector<uint64_t> hits;                 // entry id of the resident copy, 0 for a miss
    std::vector<uint64_t> evict;                // entry ids, eviction order
    std::vector<uint64_t> evict_offs;           // their offsets (for reporting)
    std::vector<Move>     moves;                // execution order
    RegionList            after;                // the Region List the commit installs
    uint64_t              reused_bytes = 0, transfer_bytes = 0, copy_bytes = 0;
    uint64_t              evicted_bytes = 0, moved_bytes = 0, merge_bound = 0;
    bool                  consumed = false;
};

struct Stats {
    uint64_t capacity, free_bytes, largest_free, n_regions, n_free_regions, n_entries, n_active,
        generation;
};

struct ModelCost { double miss_prob = 1.0, load_bw = 1.0, alpha = 1.0; };

class ReuseStore {
public:
    ReuseStore(uint64_t base_addr, uint64_t capacity, uint32_t align);

    uint64_t base() const { return base_; }
    uint64_t capacity() const { return capacity_; }
    uint32_t align() const { return align_; }
    uint64_t generation() const { return generation_; }
    uint64_t round_up(uint64_t n) const { return (n + align_ - 1) & ~uint64_t(align_ - 1); }

    bool model_active(uint64_t model_id) const;

    // Resident candidates for a key as (offset, entry id), ascending offset.
    void candidates(uint64_t fp, uint64_t nbytes, std::vector<std::pair<uint64_t, uint64_t>> &out) const;

    // Eviction, placement and (if needed) packing for tensors whose resident
    // copies (entry ids, 0 for a miss) have been chosen.  Does not modify the store.
    Status plan(const std::vector<TensorIn> &tensors, const std::vector<uint64_t> &hits, uint32_t flags,
                Plan &plan) const;

    // Install a plan made for the current generation.
    Status commit(Plan &plan, std::vector<uint64_t> &dst_offs);

    // Give up a plan whose evictions and moves have already happened to the
    // bytes in the pool: they are installed, the plan's new slots stay free.
    Status abandon(Plan &plan);

    // Remove rows whose bytes are known to be wrong (a moved tensor that no
    // longer matches its fingerprint); rows in use by a running model are kept.
    void drop_corrupt(const std::vector<uint64_t> &entry_ids);

    Status release(uint64_t model_id, bool evict);

    Status set_model_cost(uint64_t model_id, double miss_prob, double load_bw, double alpha);
    double eviction_cost(const Entry &e) const;             // Eq. 2

    uint64_t reuse_size(const std::vector<TensorIn> &tensors) const;

    Stats stats() const;
    const RegionList &region_list() const { return regions_; }
    std::vector<const Entry *> entries_by_offset() const;

private:
    struct Model { bool active = false; std::vector<uint64_t> current, owned; };

    void drop_entry(uint64_t id);      // remove from mapping and owners' lists (region handled by caller)

    uint64_t base_, capacity_;
    uint32_t align_;
    uint64_t generation_ = 0;
    uint64_t next_id_ = 1;
    RegionList regions_;
    std::unordered_map<uint64_t, Entry> entries_;                   // by entry id
    std::unordered_multimap<Key, uint64_t, KeyHash> mapping_;       // Tensor Mapping: key -> entry id
    std::unordered_map<uint64_t, Model> models_;
    std::unordered_map<uint64_t, ModelCost> costs_;
};

}  // namespace tg
