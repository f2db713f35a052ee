// Host-side Reuse Store: see reuse_store.h.
#include "reuse_store.h"

#include <algorithm>
#include <numeric>

namespace tg {

ReuseStore::ReuseStore(uint64_t base_addr, uint64_t capacity, uint32_t align)
    : base_(base_addr), capacity_(capacity), align_(align) {
    regions_[0] = Region{capacity, true};
    free_index_.insert({capacity, 0});
}

bool ReuseStore::model_active(uint64_t model_id) const {
    auto it = models_.find(model_id);
    if (it == models_.end()) return false;
    for (uint64_t off : it->second)
        if (entries_.at(off).active) return true;
    return false;
}

void ReuseStore::candidates(uint64_t fp, uint64_t nbytes, std::vector<uint64_t> &offs) const {
    offs.clear();
    auto range = mapping_.equal_range(Key{fp, nbytes});
    for (auto it = range.first; it != range.second; ++it) offs.push_back(it->second);
    std::sort(offs.begin(), offs.end());
}

// Section 3.2: the smallest free region that can hold the tensor; what is left
// of it stays free.  Tensors go in descending slot size (ties: model order),
// onto a private copy of the free index, so a failure changes nothing.
Status ReuseStore::place(const std::vector<TensorIn> &tensors, const std::vector<uint64_t> &src,
                         Plan &plan) const {
    const size_t n = tensors.size();
    std::vector<uint32_t> order(n);
    std::iota(order.begin(), order.end(), 0u);
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        return round_up(tensors[a].nbytes) > round_up(tensors[b].nbytes);
    });

    std::set<std::pair<uint64_t, uint64_t>> free_idx = free_index_;
    plan.ops.assign(n, Op{});
    plan.fps.resize(n);
    plan.place_order = order;
    plan.reused_bytes = plan.transfer_bytes = 0;
    for (uint32_t k : order) {
        const uint64_t need = round_up(tensors[k].nbytes);
        auto it = free_idx.lower_bound({need, 0});   // smallest len >= need, then lowest offset
        if (it == free_idx.end()) return ERR_NOSPACE;
        const uint64_t len = it->first, off = it->second;
        free_idx.erase(it);
        if (len > need) free_idx.insert({len - need, off + need});
        Op &op = plan.ops[k];
        op.dst_off = off;
        op.nbytes = tensors[k].nbytes;
        if (src[k] != UINT64_MAX) {
            op.kind = 0;
            op.src_off = src[k];
            plan.reused_bytes += op.nbytes;
        } else {
            op.kind = 1;
            op.src_off = tensors[k].src_off;
            plan.transfer_bytes += op.nbytes;
        }
        plan.fps[k] = tensors[k].fp;
    }
    plan.generation = generation_;
    plan.pool_tag = this;
    return OK;
}

void ReuseStore::take(uint64_t off, uint64_t need) {
    auto it = regions_.find(off);
    const uint64_t len = it->second.len;
    free_index_.erase({len, off});
    it->second = Region{need, false};
    if (len > need) {
        regions_[off + need] = Region{len - need, true};
        free_index_.insert({len - need, off + need});
    }
}

void ReuseStore::give(uint64_t off) {
    auto it = regions_.find(off);
    it->second.free = true;
    auto next = std::next(it);
    if (next != regions_.end() && next->second.free) {
        free_index_.erase({next->second.len, next->first});
        it->second.len += next->second.len;
        regions_.erase(next);
    }
    if (it != regions_.begin()) {
        auto prev = std::prev(it);
        if (prev->second.free) {
            free_index_.erase({prev->second.len, prev->first});
            prev->second.len += it->second.len;
            regions_.erase(it);
            it = prev;
        }
    }
    free_index_.insert({it->second.len, it->first});
}

// Section 3.1: after loading, the mapping is updated and every tensor's
// address is returned.
Status ReuseStore::commit(Plan &plan, std::vector<uint64_t> &dst_offs) {
    if (plan.consumed || plan.pool_tag != this) return ERR_INVALID;
    if (plan.generation != generation_) return ERR_STALE;
    if (model_active(plan.model_id)) return ERR_INVALID;
    // Slots are taken in the order they were planned, so each destination is
    // the start of a free region at the moment it is carved.
    for (uint32_t k : plan.place_order) {
        const Op &op = plan.ops[k];
        take(op.dst_off, round_up(op.nbytes));
    }
    auto &mine = models_[plan.model_id];
    dst_offs.resize(plan.ops.size());
    for (size_t k = 0; k < plan.ops.size(); ++k) {
        const Op &op = plan.ops[k];
        entries_[op.dst_off] = Entry{op.dst_off, op.nbytes, plan.fps[k], plan.model_id, true};
        mapping_.insert({Key{plan.fps[k], op.nbytes}, op.dst_off});
        mine.push_back(op.dst_off);
        dst_offs[k] = op.dst_off;
    }
    plan.consumed = true;
    ++generation_;
    return OK;
}

Status ReuseStore::release(uint64_t model_id, bool evict) {
    auto it = models_.find(model_id);
    if (it == models_.end()) return ERR_NOTFOUND;
    if (!evict) {
        for (uint64_t off : it->second) entries_.at(off).active = false;
    } else {
        for (uint64_t off : it->second) {
            const Entry &e = entries_.at(off);
            auto range = mapping_.equal_range(Key{e.fp, e.nbytes});
            for (auto m = range.first; m != range.second; ++m)
                if (m->second == off) { mapping_.erase(m); break; }
            entries_.erase(off);
            give(off);
        }
        models_.erase(it);
    }
    ++generation_;
    return OK;
}

uint64_t ReuseStore::reuse_size(const std::vector<TensorIn> &tensors) const {
    uint64_t total = 0;
    for (const TensorIn &t : tensors)
        if (mapping_.find(Key{t.fp, t.nbytes}) != mapping_.end()) total += t.nbytes;
    return total;
}

Stats ReuseStore::stats() const {
    Stats s{};
    s.capacity = capacity_;
    s.n_regions = regions_.size();
    s.n_free_regions = free_index_.size();
    for (const auto &f : free_index_) s.free_bytes += f.first;
    s.largest_free = free_index_.empty() ? 0 : free_index_.rbegin()->first;
    s.n_entries = entries_.size();
    for (const auto &e : entries_) s.n_active += e.second.active ? 1 : 0;
    s.generation = generation_;
    return s;
}

}  // namespace tg
