// Host-side Reuse Store: see reuse_store.h.
#include "reuse_store.h"

#include <algorithm>
#include <iterator>
#include <numeric>

namespace tg {

// ------------------------------------------------------------------ RegionList
RegionList::RegionList(uint64_t capacity) {
    by_off_[0] = Region{capacity, true, 0};
    free_idx_.insert({capacity, 0});
    free_bytes_ = capacity;
}

// Section 3.2: the smallest free region that can hold the tensor (ties: lowest offset).
bool RegionList::best_fit(uint64_t need, uint64_t &off) const {
    auto it = free_idx_.lower_bound({need, 0});
    if (it == free_idx_.end()) return false;
    off = it->second;
    return true;
}

// Section 3.2: what is left of the free region stays free.
void RegionList::take(uint64_t off, uint64_t need, uint64_t tag) {
    auto it = by_off_.find(off);
    const uint64_t len = it->second.len;
    free_idx_.erase({len, off});
    it->second = Region{need, false, tag};
    if (len > need) {
        by_off_[off + need] = Region{len - need, true, 0};
        free_idx_.insert({len - need, off + need});
    }
    free_bytes_ -= need;
}

void RegionList::give(uint64_t off) {
    auto it = by_off_.find(off);
    it->second.free = true;
    it->second.tag = 0;
    free_bytes_ += it->second.len;
    auto next = std::next(it);
    if (next != by_off_.end() && next->second.free) {
        free_idx_.erase({next->second.len, next->first});
        it->second.len += next->second.len;
        by_off_.erase(next);
    }
    if (it != by_off_.begin()) {
        auto prev = std::prev(it);
        if (prev->second.free) {
            free_idx_.erase({prev->second.len, prev->first});
            prev->second.len += it->second.len;
            by_off_.erase(it);
            it = prev;
        }
    }
    free_idx_.insert({it->second.len, it->first});
}

std::vector<RegionList::Flat> RegionList::flatten() const {
    std::vector<Flat> out;
    out.reserve(by_off_.size());
    for (const auto &r : by_off_) out.push_back(Flat{r.first, r.second.len, r.second.free, r.second.tag});
    return out;
}

void RegionList::rebuild(const std::vector<Flat> &flat) {
    by_off_.clear();
    free_idx_.clear();
    free_bytes_ = 0;
    for (const Flat &f : flat) {
        by_off_.emplace_hint(by_off_.end(), f.off, Region{f.len, f.free, f.tag});
        if (f.free) {
            free_idx_.insert({f.len, f.off});
            free_bytes_ += f.len;
        }
    }
}

// ------------------------------------------------------------------ Algorithm 1
namespace {

using Flat = RegionList::Flat;
struct Range { size_t lo = 0, hi = 0; bool ok = false; };

// Largest sub-range of regs[lo, hi) that begins and ends with a free region.
Range trim(const std::vector<Flat> &regs, size_t lo, size_t hi) {
    while (lo < hi && !regs[lo].free) ++lo;
    while (hi > lo && !regs[hi - 1].free) --hi;
    Range r;
    r.lo = lo;
    r.hi = hi;
    r.ok = lo < hi;
    return r;
}

uint64_t free_bytes_of(const std::vector<Flat> &regs, const Range &r) {
    uint64_t f = 0;
    if (r.ok)
        for (size_t i = r.lo; i < r.hi; ++i)
            if (regs[i].free) f += regs[i].len;
    return f;
}

// TryPacking of Algorithm 1, as listed: tensors in descending size go to the
// bin with more remaining capacity; fail as soon as one is not smaller than
// the smaller remaining capacity.  Both outputs empty = failure.
void try_packing(const std::vector<uint64_t> &sizes, const std::vector<uint32_t> &tensors, uint64_t c1,
                 uint64_t c2, std::vector<uint32_t> &t1, std::vector<uint32_t> &t2) {
    t1.clear();
    t2.clear();
    for (uint32_t k : tensors) {
        if (sizes[k] >= std::min(c1, c2)) {
            t1.clear();
            t2.clear();
            return;
        }
        if (c1 >= c2) { t1.push_back(k); c1 -= sizes[k]; }
        else          { t2.push_back(k); c2 -= sizes[k]; }
    }
}

// Either side of a region that cannot move: a tensor goes to the side with
// more room and only has to fit there.  (Not part of Algorithm 1.)
bool split_at_wall(const std::vector<uint64_t> &sizes, const std::vector<uint32_t> &tensors, uint64_t c1,
                   uint64_t c2, std::vector<uint32_t> &t1, std::vector<uint32_t> &t2) {
    t1.clear();
    t2.clear();
    for (uint32_t k : tensors) {
        if (c1 >= c2) {
            if (sizes[k] > c1) return false;
            t1.push_back(k);
            c1 -= sizes[k];
        } else {
            if (sizes[k] > c2) return false;
            t2.push_back(k);
            c2 -= sizes[k];
        }
    }
    return true;
}

// Algorithm 1.  `movable[i]` says whether allocated region i may move.
// Returns false when immovable regions keep the tensors from being split.
bool partitioned_gain_packing(const std::vector<Flat> &regs, const std::vector<uint64_t> &sizes,
                              const std::vector<uint32_t> &order, const std::vector<char> &movable,
                              bool pack_text, std::vector<Subspace> &final_set, uint64_t &merge_cost) {
    final_set.clear();
    Range whole = trim(regs, 0, regs.size());
    if (!whole.ok) return false;
    std::vector<Subspace> pending;
    std::vector<uint32_t> t1, t2;
    {
        Range sub = whole;
        std::vector<uint32_t> tensors = order;
        for (;;) {
            size_t wall = sub.hi;
            for (size_t i = sub.lo; i < sub.hi; ++i)
                if (!regs[i].free && !movable[i]) { wall = i; break; }
            if (wall == sub.hi) {
                pending.push_back(Subspace{sub.lo, sub.hi, tensors});
                break;
            }
            const Range p1 = trim(regs, sub.lo, wall), p2 = trim(regs, wall + 1, sub.hi);
            if (!split_at_wall(sizes, tensors, free_bytes_of(regs, p1), free_bytes_of(regs, p2), t1, t2))
                return false;
            if (p1.ok) pending.push_back(Subspace{p1.lo, p1.hi, t1});
            else if (!t1.empty()) return false;
            if (!p2.ok) {
                if (!t2.empty()) return false;
                break;
            }
            sub = p2;
            tensors = t2;
        }
    }
    merge_cost = 0;
    for (const Subspace &s : pending)
        for (size_t i = s.lo; i < s.hi; ++i)
            if (!regs[i].free) merge_cost += regs[i].len;

    std::vector<size_t> points;
    while (!pending.empty()) {
        std::vector<Subspace> next;
        for (Subspace &s : pending) {
            points.clear();
            for (size_t i = s.lo; i < s.hi; ++i)
                if (!regs[i].free) points.push_back(i);
            // the partition gain of a point is its size: largest first, ties by offset
            std::stable_sort(points.begin(), points.end(),
                             [&](size_t a, size_t b) { return regs[a].len > regs[b].len; });
            bool split = false;
            for (size_t p : points) {
                const Range p1 = trim(regs, s.lo, p), p2 = trim(regs, p + 1, s.hi);
                // the listing's test, or the one the text words (a tensor only has to fit
                // the bin with more room)
                if (!pack_text) {
                    try_packing(sizes, s.tensors, free_bytes_of(regs, p1), free_bytes_of(regs, p2), t1, t2);
                } else if (!split_at_wall(sizes, s.tensors, free_bytes_of(regs, p1), free_bytes_of(regs, p2), t1, t2)) {
                    t1.clear();
                    t2.clear();
                }
                if (!t1.empty() || !t2.empty()) {
                    if (p1.ok) next.push_back(Subspace{p1.lo, p1.hi, t1});
                    if (p2.ok) next.push_back(Subspace{p2.lo, p2.hi, t2});
                    merge_cost -= regs[p].len;
                    split = true;
                    break;
                }
            }
            if (!split) final_set.push_back(std::move(s));
        }
        pending.swap(next);
    }
    std::sort(final_set.begin(), final_set.end(),
              [](const Subspace &a, const Subspace &b) { return a.lo < b.lo; });
    return true;
}

// Best fit restricted to a flat list (one subspace); carves like RegionList::take.
bool best_fit_flat(std::vector<Flat> &part, uint64_t need, uint64_t tag, uint64_t &off) {
    size_t pick = part.size();
    for (size_t i = 0; i < part.size(); ++i) {
        if (!part[i].free || part[i].len < need) continue;
        if (pick == part.size() || part[i].len < part[pick].len) pick = i;
    }
    if (pick == part.size()) return false;
    off = part[pick].off;
    const uint64_t len = part[pick].len;
    part[pick] = Flat{off, need, false, tag};
    if (len > need) part.insert(part.begin() + pick + 1, Flat{off + need, len - need, true, 0});
    return true;
}

}  // namespace

// ------------------------------------------------------------------ ReuseStore
ReuseStore::ReuseStore(uint64_t base_addr, uint64_t capacity, uint32_t align)
    : base_(base_addr), capacity_(capacity), align_(align), regions_(capacity) {}

bool ReuseStore::model_active(uint64_t model_id) const {
    auto it = models_.find(model_id);
    return it != models_.end() && it->second.active;
}

void ReuseStore::candidates(uint64_t fp, uint64_t nbytes,
                            std::vector<std::pair<uint64_t, uint64_t>> &out) const {
    out.clear();
    auto range = mapping_.equal_range(Key{fp, nbytes});
    for (auto it = range.first; it != range.second; ++it)
        out.push_back({entries_.at(it->second).off, it->second});
    std::sort(out.begin(), out.end());
}

Status ReuseStore::set_model_cost(uint64_t model_id, double miss_prob, double load_bw, double alpha) {
    if (!(miss_prob >= 0.0) || !(load_bw > 0.0) || !(alpha >= 0.0)) return ERR_INVALID;
    costs_[model_id] = ModelCost{miss_prob, load_bw, alpha};
    return OK;
}

// Eq. 2: c_j = p_m * (s'_j / b_m) * alpha_m; a tensor several models own costs
// the sum over its owners.  No contraction, so the value is the same double
// any other IEEE evaluation of this expression gives.
#pragma clang fp contract(off)
double ReuseStore::eviction_cost(const Entry &e) const {
    double total = 0.0;
    for (uint64_t m : e.owners) {
        ModelCost c;
        auto it = costs_.find(m);
        if (it != costs_.end()) c = it->second;
        const double per_byte_time = double(e.nbytes) / c.load_bw;
        const double weighted = c.miss_prob * per_byte_time;
        total = total + weighted * c.alpha;
    }
    return total;
}

Status ReuseStore::plan(const std::vector<TensorIn> &tensors, const std::vector<uint64_t> &hits,
                        uint32_t flags, Plan &plan) const {
    const size_t n = tensors.size();
    const bool alias = (flags & PLAN_ALIAS) != 0;
    plan.alias = alias;
    plan.hits = hits;
    plan.fps.resize(n);
    plan.ops.assign(n, Op{});
    plan.evict.clear();
    plan.evict_offs.clear();
    plan.moves.clear();
    plan.evicted_bytes = plan.moved_bytes = plan.merge_bound = 0;

    std::vector<uint64_t> sizes(n);
    std::vector<uint32_t> order;
    uint64_t need_total = 0;
    for (size_t k = 0; k < n; ++k) {
        sizes[k] = round_up(tensors[k].nbytes);
        plan.fps[k] = tensors[k].fp;
        if (!(alias && hits[k] != 0)) {
            order.push_back(uint32_t(k));
            need_total += sizes[k];
        }
    }
    // descending slot size, ties by index (Algorithm 1's input convention)
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t a, uint32_t b) { return sizes[a] > sizes[b]; });

    RegionList work = regions_;

    // ---- Stage 1: minimal-cost eviction (Section 3.2, Eq. 2)
    if ((flags & PLAN_EVICT) && work.free_bytes() < need_total) {
        std::set<uint64_t> keep(hits.begin(), hits.end());
        struct Cand { double cost; uint64_t off, id; };
        std::vector<Cand> cands;
        for (const auto &kv : entries_) {
            const Entry &e = kv.second;
            if (e.active_refs != 0 || keep.count(e.id)) continue;
            cands.push_back(Cand{eviction_cost(e), e.off, e.id});
        }
        std::sort(cands.begin(), cands.end(), [](const Cand &a, const Cand &b) {
            return a.cost < b.cost || (a.cost == b.cost && a.off < b.off);
        });
        for (const Cand &c : cands) {
            if (work.free_bytes() >= need_total) break;
            work.give(c.off);
            plan.evict.push_back(c.id);
            plan.evict_offs.push_back(c.off);
            plan.evicted_bytes += round_up(entries_.at(c.id).nbytes);
        }
    }
    if (work.free_bytes() < need_total) return ERR_NOSPACE;

    // ---- best fit (Section 3.2)
    std::vector<uint64_t> dst(n, 0);
    {
        RegionList trial = work;
        bool ok = true;
        for (uint32_t k : order) {
            uint64_t off;
            if (!trial.best_fit(sizes[k], off)) { ok = false; break; }
            trial.take(off, sizes[k], kNewTag + k);
            dst[k] = off;
        }
        if (ok) {
            work = std::move(trial);
        } else if (!(flags & PLAN_MERGE)) {
            return ERR_NOSPACE;
        } else {
            // ---- Stage 2: Partitioned-Gain Packing (Algorithm 1)
            std::vector<Flat> regs = work.flatten();
            std::vector<char> movable(regs.size(), 0);
            for (size_t i = 0; i < regs.size(); ++i)
                if (!regs[i].free) movable[i] = entries_.at(regs[i].tag).active_refs == 0;
            std::vector<Subspace> final_set;
            if (!partitioned_gain_packing(regs, sizes, order, movable, (flags & PLAN_PACK_TEXT) != 0, final_set,
                                          plan.merge_bound))
                return ERR_NOSPACE;
            // realise the subspaces; the flat list is rebuilt piece by piece in address order
            std::vector<Flat> out;
            out.reserve(regs.size() + n);
            size_t at_index = 0;
            for (const Subspace &s : final_set) {
                for (; at_index < s.lo; ++at_index) out.push_back(regs[at_index]);
                std::vector<Flat> part(regs.begin() + s.lo, regs.begin() + s.hi);
                std::vector<Flat> trial_part = part;
                bool fits = true;
                for (uint32_t k : s.tensors) {
                    uint64_t off;
                    if (!best_fit_flat(trial_part, sizes[k], kNewTag + k, off)) { fits = false; break; }
                    dst[k] = off;
                }
                if (fits) {
                    part.swap(trial_part);
                } else {
                    // merge: slide every allocated region to the subspace's low end in
                    // address order, then place the tensors in the free tail
                    const uint64_t start = part.front().off;
                    const uint64_t end = part.back().off + part.back().len;
                    uint64_t at = start;
                    std::vector<Flat> packed;
                    for (const Flat &r : part) {
                        if (r.free) continue;
                        if (r.off != at) {
                            const Entry &e = entries_.at(r.tag);
                            plan.moves.push_back(Move{e.id, r.off, at, e.nbytes, e.fp});
                            plan.moved_bytes += e.nbytes;
                        }
                        packed.push_back(Flat{at, r.len, false, r.tag});
                        at += r.len;
                    }
                    for (uint32_t k : s.tensors) {
                        dst[k] = at;
                        packed.push_back(Flat{at, sizes[k], false, kNewTag + k});
                        at += sizes[k];
                    }
                    if (at > end) return ERR_NOSPACE;      // cannot happen: packing respects free bytes
                    if (at < end) packed.push_back(Flat{at, end - at, true, 0});
                    part.swap(packed);
                }
                out.insert(out.end(), part.begin(), part.end());
                at_index = s.hi;
            }
            for (; at_index < regs.size(); ++at_index) out.push_back(regs[at_index]);
            work.rebuild(out);
        }
    }

    std::unordered_map<uint64_t, uint64_t> moved_to;
    for (const Move &m : plan.moves) moved_to[m.entry] = m.new_off;
    plan.reused_bytes = plan.transfer_bytes = plan.copy_bytes = 0;
    for (size_t k = 0; k < n; ++k) {
        Op &op = plan.ops[k];
        op.nbytes = tensors[k].nbytes;
        if (hits[k] == 0) {
            op.kind = 1;
            op.dst_off = dst[k];
            op.src_off = tensors[k].src_off;
            plan.transfer_bytes += op.nbytes;
        } else {
            auto mv = moved_to.find(hits[k]);
            const uint64_t where = mv != moved_to.end() ? mv->second : entries_.at(hits[k]).off;
            op.kind = 0;
            op.src_off = where;
            op.dst_off = alias ? where : dst[k];
            plan.reused_bytes += op.nbytes;
            if (!alias) plan.copy_bytes += op.nbytes;
        }
    }
    plan.after = std::move(work);
    plan.generation = generation_;
    plan.pool_tag = this;
    plan.consumed = false;
    return OK;
}

void ReuseStore::drop_entry(uint64_t id) {
    Entry &e = entries_.at(id);
    auto range = mapping_.equal_range(Key{e.fp, e.nbytes});
    for (auto m = range.first; m != range.second; ++m)
        if (m->second == id) { mapping_.erase(m); break; }
    for (uint64_t mid : e.owners) {
        auto it = models_.find(mid);
        if (it == models_.end()) continue;
        auto &owned = it->second.owned;
        owned.erase(std::remove(owned.begin(), owned.end(), id), owned.end());
        auto &cur = it->second.current;
        cur.erase(std::remove(cur.begin(), cur.end(), id), cur.end());
        if (owned.empty()) models_.erase(it);
    }
    entries_.erase(id);
}

// Section 3.1: after loading, the mapping is updated and every tensor's
// address is returned.
Status ReuseStore::commit(Plan &plan, std::vector<uint64_t> &dst_offs) {
    if (plan.consumed || plan.pool_tag != this) return ERR_INVALID;
    if (plan.generation != generation_) return ERR_STALE;
    if (model_active(plan.model_id)) return ERR_INVALID;

    for (uint64_t id : plan.evict) drop_entry(id);
    for (const Move &m : plan.moves) entries_.at(m.entry).off = m.new_off;
    regions_ = std::move(plan.after);

    Model &model = models_[plan.model_id];
    model.active = true;
    dst_offs.resize(plan.ops.size());
    for (size_t k = 0; k < plan.ops.size(); ++k) {
        const Op &op = plan.ops[k];
        uint64_t id;
        if (plan.alias && plan.hits[k] != 0) {
            id = plan.hits[k];
            Entry &e = entries_.at(id);
            if (std::find(e.owners.begin(), e.owners.end(), plan.model_id) == e.owners.end())
                e.owners.push_back(plan.model_id);
        } else {
            id = next_id_++;
            Entry e;
            e.id = id;
            e.off = op.dst_off;
            e.nbytes = op.nbytes;
            e.fp = plan.fps[k];
            e.owners.push_back(plan.model_id);
            entries_.emplace(id, std::move(e));
            mapping_.insert({Key{plan.fps[k], op.nbytes}, id});
            regions_.set_tag(op.dst_off, id);
        }
        if (std::find(model.current.begin(), model.current.end(), id) == model.current.end()) {
            model.current.push_back(id);
            entries_.at(id).active_refs += 1;
        }
        if (std::find(model.owned.begin(), model.owned.end(), id) == model.owned.end())
            model.owned.push_back(id);
        dst_offs[k] = op.dst_off;
    }
    plan.consumed = true;
    ++generation_;
    return OK;
}

// A plan that stopped half way: what it evicted has been overwritten and what
// it moved lies at its new address, so both are recorded; the slots it meant
// to fill go back to the free regions and the model gains nothing.
Status ReuseStore::abandon(Plan &plan) {
    if (plan.consumed || plan.pool_tag != this) return ERR_INVALID;
    if (plan.generation != generation_) return ERR_STALE;
    for (uint64_t id : plan.evict) drop_entry(id);
    for (const Move &m : plan.moves) entries_.at(m.entry).off = m.new_off;
    regions_ = std::move(plan.after);
    for (size_t k = 0; k < plan.ops.size(); ++k)
        if (!(plan.alias && plan.hits[k] != 0)) regions_.give(plan.ops[k].dst_off);
    plan.consumed = true;
    ++generation_;
    return OK;
}

void ReuseStore::drop_corrupt(const std::vector<uint64_t> &entry_ids) {
    bool any = false;
    for (uint64_t id : entry_ids) {
        auto it = entries_.find(id);
        if (it == entries_.end() || it->second.active_refs != 0) continue;
        const uint64_t off = it->second.off;
        drop_entry(id);
        regions_.give(off);
        any = true;
    }
    if (any) ++generation_;
}

Status ReuseStore::release(uint64_t model_id, bool evict) {
    auto it = models_.find(model_id);
    if (it == models_.end()) return ERR_NOTFOUND;
    Model &m = it->second;
    for (uint64_t id : m.current) entries_.at(id).active_refs -= 1;
    m.current.clear();
    m.active = false;
    if (evict) {
        const std::vector<uint64_t> owned = m.owned;
        for (uint64_t id : owned) {
            Entry &e = entries_.at(id);
            e.owners.erase(std::remove(e.owners.begin(), e.owners.end(), model_id), e.owners.end());
            if (e.owners.empty()) {
                const uint64_t off = e.off;
                auto range = mapping_.equal_range(Key{e.fp, e.nbytes});
                for (auto mm = range.first; mm != range.second; ++mm)
                    if (mm->second == id) { mapping_.erase(mm); break; }
                entries_.erase(id);
                regions_.give(off);
            }
        }
        models_.erase(model_id);
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

std::vector<const Entry *> ReuseStore::entries_by_offset() const {
    std::vector<const Entry *> out;
    out.reserve(entries_.size());
    for (const auto &kv : entries_) out.push_back(&kv.second);
    std::sort(out.begin(), out.end(), [](const Entry *a, const Entry *b) { return a->off < b->off; });
    return out;
}

Stats ReuseStore::stats() const {
    Stats s{};
    s.capacity = capacity_;
    s.n_regions = regions_.size();
    s.n_free_regions = regions_.n_free();
    s.free_bytes = regions_.free_bytes();
    s.largest_free = regions_.largest_free();
    s.n_entries = entries_.size();
    for (const auto &e : entries_) s.n_active += e.second.active_refs > 0 ? 1 : 0;
    s.generation = generation_;
    return s;
}

}  // namespace tg
