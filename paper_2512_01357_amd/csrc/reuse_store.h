// Host-side Reuse Store: Region List, Tensor Mapping and the load planner.
//
// Pure C++ (no HIP): everything here runs on the CPU and decides *what* the
// device will be asked to do.  Follows the paper's Section 3.1 (Tensor
// Mapping lookup, return addresses) and Section 3.2 (regions in physical
// order, best-fit allocation).
#pragma once

#include <cstdint>
#include <map>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

namespace tg {

struct Entry {            // one row of the Tensor Mapping
    uint64_t off;         // slot offset in the pool
    uint64_t nbytes;      // tensor length (slot is roundup(nbytes, align))
    uint64_t fp;
    uint64_t model_id;
    bool     active;
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

struct TensorIn {         // one incoming tensor
    uint64_t nbytes, fp, src_off;
};

struct Op {               // decision for one incoming tensor
    uint32_t kind;        // 0 reuse, 1 host-to-device
    uint64_t dst_off, src_off, nbytes;
};

struct Plan {
    uint64_t              model_id = 0;
    const void           *host_base = nullptr;
    uint64_t              host_bytes = 0;
    uint64_t              generation = 0;
    const void           *pool_tag = nullptr;   // the pool the plan was made for
    std::vector<Op>       ops;                  // model order
    std::vector<uint64_t> fps;                  // model order
    std::vector<uint32_t> place_order;          // order in which slots were taken
    uint64_t              reused_bytes = 0, transfer_bytes = 0;
    bool                  consumed = false;
};

struct Stats {
    uint64_t capacity, free_bytes, largest_free, n_regions, n_free_regions, n_entries, n_active,
        generation;
};

enum Status : int32_t {
    OK = 0, ERR_INVALID = -1, ERR_NOSPACE = -2, ERR_STALE = -3, ERR_NOTFOUND = -4, ERR_HIP = -5,
    ERR_NOMEM = -6, ERR_CORRUPT = -7
};

class ReuseStore {
public:
    ReuseStore(uint64_t base_addr, uint64_t capacity, uint32_t align);

    uint64_t base() const { return base_; }
    uint64_t capacity() const { return capacity_; }
    uint32_t align() const { return align_; }
    uint64_t generation() const { return generation_; }
    uint64_t round_up(uint64_t n) const { return (n + align_ - 1) & ~uint64_t(align_ - 1); }

    bool model_active(uint64_t model_id) const;

    // Resident candidates for a key, ascending pool offset.
    void candidates(uint64_t fp, uint64_t nbytes, std::vector<uint64_t> &offs) const;

    // Best-fit placement of every tensor on a copy of the free index.
    // `src` holds, per tensor, the reuse source offset or UINT64_MAX for a miss.
    Status place(const std::vector<TensorIn> &tensors, const std::vector<uint64_t> &src, Plan &plan) const;

    // Install a plan made for the current generation.
    Status commit(Plan &plan, std::vector<uint64_t> &dst_offs);

    Status release(uint64_t model_id, bool evict);

    uint64_t reuse_size(const std::vector<TensorIn> &tensors) const;

    Stats stats() const;

private:
    struct Region { uint64_t len; bool free; };

    void take(uint64_t off, uint64_t need);   // carve [off, off+need) from the free region starting at off
    void give(uint64_t off);                  // free the allocated region at off and merge neighbours

    uint64_t base_, capacity_;
    uint32_t align_;
    uint64_t generation_ = 0;
    std::map<uint64_t, Region>                 regions_;     // by offset: the Region List
    std::set<std::pair<uint64_t, uint64_t>>    free_index_;  // (len, off): best-fit = lower_bound
    std::unordered_map<uint64_t, Entry>        entries_;     // by slot offset
    std::unordered_multimap<Key, uint64_t, KeyHash> mapping_; // Tensor Mapping: key -> slot offset
    std::unordered_map<uint64_t, std::vector<uint64_t>> models_; // model id -> slot offsets
};

}  // namespace tg
