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

// Replaces the regions that tile [start, end) by `flats` (which tile the same bytes).
void RegionList::splice(uint64_t start, uint64_t end, const std::vector<Flat> &flats) {
    auto it = by_off_.lower_bound(start);
    while (it != by_off_.end() && it->first < end) {
        if (it->second.free) {
            free_idx_.erase({it->second.len, it->first});
            free_bytes_ -= it->second.len;
        }
        it = by_off_.erase(it);
    }
    for (const Flat &f : flats) {
        by_off_.emplace_hint(it, f.off, Region{f.len, f.free, f.tag});
        if (f.free) {
            free_idx_.insert({f.len, f.off});
            free_bytes_ += f.len;
        }
    }
}

// ------------------------------------------------------------------ Stage 2
namespace {

using Flat = RegionList::Flat;

// Partitioned-Gain Packing (Section 3.2, Algorithm 1) over a snapshot of the
// Region List.  Regions are addressed by index; byte counts of any index range
// come from prefix sums, the subspace inside a range (its first to its last free
// region) from two look-up arrays, so a partition attempt costs one pass over
// the tensors and nothing over the regions.
class Packer {
public:
    struct Piece { size_t lo, hi; std::vector<uint32_t> tensors; };      // regions [lo, hi) and what goes there

    Packer(const std::vector<Flat> &regs, const std::vector<uint64_t> &sizes, bool pack_text, bool cap_text)
        : regs_(regs), sizes_(sizes), pack_text_(pack_text), cap_text_(cap_text) {
        const size_t n = regs.size();
        free_before_.assign(n + 1, 0);
        used_before_.assign(n + 1, 0);
        free_at_or_after_.assign(n + 1, n);
        free_at_or_before_.assign(n + 1, n);
        for (size_t i = 0; i < n; ++i) {
            free_before_[i + 1] = free_before_[i] + (regs[i].free ? regs[i].len : 0);
            used_before_[i + 1] = used_before_[i] + (regs[i].free ? 0 : regs[i].len);
        }
        for (size_t i = n; i-- > 0;) free_at_or_after_[i] = regs[i].free ? i : free_at_or_after_[i + 1];
        for (size_t i = 0; i < n; ++i) free_at_or_before_[i] = regs[i].free ? i : (i ? free_at_or_before_[i - 1] : n);
    }

    uint64_t free_bytes(size_t lo, size_t hi) const { return free_before_[hi] - free_before_[lo]; }
    uint64_t used_bytes(size_t lo, size_t hi) const { return used_before_[hi] - used_before_[lo]; }

    // The subspace inside [lo, hi): from its first to its last free region.  False if it has none.
    bool narrow(size_t &lo, size_t &hi) const {
        if (lo >= hi) return false;
        const size_t first = free_at_or_after_[lo], last = free_at_or_before_[hi - 1];
        if (first >= hi || last == regs_.size() || last < lo) return false;
        lo = first;
        hi = last + 1;
        return true;
    }

    // What a range can be given: its free bytes, or free plus allocated bytes under the text's definition.
    uint64_t room(bool ok, size_t lo, size_t hi) const {
        if (!ok) return 0;
        return free_bytes(lo, hi) + (cap_text_ ? used_bytes(lo, hi) : 0);
    }

    // Deals `tensors` (descending size) over two bins of room a and b: each goes to the bin with
    // more room left (the first on ties).  side[i] = 0 or 1.  The listing refuses a tensor that is
    // not smaller than the smaller bin's room; the text only one that does not fit its own bin.
    bool two_bins(const std::vector<uint32_t> &tensors, uint64_t a, uint64_t b, std::vector<uint8_t> &side) const {
        side.resize(tensors.size());
        for (size_t i = 0; i < tensors.size(); ++i) {
            const uint64_t need = sizes_[tensors[i]];
            const bool second = a < b;
            const bool refused = pack_text_ ? need > (second ? b : a) : need >= (second ? a : b);
            if (refused) return false;
            side[i] = second ? 1 : 0;
            (second ? b : a) -= need;
        }
        return true;
    }

    // Starting pairs: the pool cut at every region that may not move; the tensors go to the
    // piece with the most room left (lowest address on ties).  False if one fits nowhere.
    bool deal(const std::vector<uint32_t> &order, const std::vector<char> &movable, std::vector<Piece> &out) const {
        out.clear();
        size_t lo = 0;
        for (size_t i = 0; i <= regs_.size(); ++i) {
            if (i < regs_.size() && (regs_[i].free || movable[i])) continue;
            size_t a = lo, b = i;
            if (narrow(a, b)) out.push_back(Piece{a, b, {}});
            lo = i + 1;
        }
        std::vector<uint64_t> left(out.size());
        for (size_t j = 0; j < out.size(); ++j) left[j] = room(true, out[j].lo, out[j].hi);
        for (uint32_t k : order) {
            if (out.empty()) return false;
            size_t best = 0;
            for (size_t j = 1; j < out.size(); ++j)
                if (left[j] > left[best]) best = j;
            if (sizes_[k] > left[best]) return false;
            out[best].tensors.push_back(k);
            left[best] -= sizes_[k];
        }
        return true;
    }

    // Algorithm 1 on the starting pairs.  Pieces come back in address order, those without tensors
    // left out.  A piece is cut at the largest allocated region (lowest address on ties) at which
    // its tensors can be dealt over the two sides; what cannot be cut is final.
    std::vector<Piece> run(std::vector<Piece> todo) const {
        std::vector<Piece> done;
        std::vector<size_t> points;
        std::vector<uint8_t> side;
        while (!todo.empty()) {
            Piece cur = std::move(todo.back());
            todo.pop_back();
            if (cur.tensors.empty()) continue;                    // nothing to place: nothing to merge
            points.clear();
            for (size_t i = cur.lo; i < cur.hi; ++i)
                if (!regs_[i].free) points.push_back(i);
            std::stable_sort(points.begin(), points.end(),
                             [&](size_t x, size_t y) { return regs_[x].len > regs_[y].len; });
            bool cut = false;
            for (size_t p : points) {
                size_t l0 = cur.lo, l1 = p, r0 = p + 1, r1 = cur.hi;
                const bool lok = narrow(l0, l1), rok = narrow(r0, r1);
                if (!two_bins(cur.tensors, room(lok, l0, l1), room(rok, r0, r1), side)) continue;
                Piece left{l0, l1, {}}, right{r0, r1, {}};
                for (size_t i = 0; i < cur.tensors.size(); ++i) (side[i] ? right : left).tensors.push_back(cur.tensors[i]);
                todo.push_back(std::move(left));
                todo.push_back(std::move(right));
                cut = true;
                break;
            }
            if (!cut) done.push_back(std::move(cur));
        }
        std::sort(done.begin(), done.end(), [](const Piece &a, const Piece &b) { return a.lo < b.lo; });
        return done;
    }

private:
    const std::vector<Flat> &regs_;
    const std::vector<uint64_t> &sizes_;
    const bool pack_text_, cap_text_;
    std::vector<uint64_t> free_before_, used_before_;
    std::vector<size_t> free_at_or_after_, free_at_or_before_;
};

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
            const std::vector<Flat> regs = work.flatten();
            std::vector<char> movable(regs.size(), 0);
            for (size_t i = 0; i < regs.size(); ++i)
                if (!regs[i].free) movable[i] = entries_.at(regs[i].tag).active_refs == 0;
            const Packer packer(regs, sizes, (flags & PLAN_PACK_TEXT) != 0, (flags & PLAN_CAP_TEXT) != 0);
            std::vector<Packer::Piece> start;
            if (!packer.deal(order, movable, start)) return ERR_NOSPACE;
            const std::vector<Packer::Piece> pieces = packer.run(std::move(start));
            for (const Packer::Piece &pc : pieces) {
                // only residents inside a piece that takes tensors can ever move
                plan.merge_bound += packer.used_bytes(pc.lo, pc.hi);
                uint64_t need = 0;
                for (uint32_t k : pc.tensors) need += sizes[k];
                // cannot happen by free bytes; the text's capacity counts allocated bytes as room
                if (need > packer.free_bytes(pc.lo, pc.hi)) return ERR_NOSPACE;
            }
            for (const Packer::Piece &pc : pieces) {
                const uint64_t begin = regs[pc.lo].off, end = regs[pc.hi - 1].off + regs[pc.hi - 1].len;
                // best fit restricted to the piece: its holes by (length, offset)
                std::set<std::pair<uint64_t, uint64_t>> holes;
                for (size_t i = pc.lo; i < pc.hi; ++i)
                    if (regs[i].free) holes.insert({regs[i].len, regs[i].off});
                std::vector<std::pair<uint32_t, uint64_t>> placed;
                for (uint32_t k : pc.tensors) {
                    auto h = holes.lower_bound({sizes[k], 0});
                    if (h == holes.end()) break;
                    const uint64_t len = h->first, off = h->second;
                    holes.erase(h);
                    if (len > sizes[k]) holes.insert({len - sizes[k], off + sizes[k]});
                    placed.push_back({k, off});
                }
                if (placed.size() == pc.tensors.size()) {
                    for (const auto &kd : placed) {               // same order, so each hole is carved the same way
                        work.take(kd.second, sizes[kd.first], kNewTag + kd.first);
                        dst[kd.first] = kd.second;
                    }
                    continue;
                }
                // merge: the residents slide to the piece's low end in address order, the
                // tensors follow, what is left is one free region
                std::vector<Flat> packed;
                uint64_t at = begin;
                for (size_t i = pc.lo; i < pc.hi; ++i) {
                    if (regs[i].free) continue;
                    if (regs[i].off != at) {
                        const Entry &e = entries_.at(regs[i].tag);
                        plan.moves.push_back(Move{e.id, regs[i].off, at, e.nbytes, e.fp});
                        plan.moved_bytes += e.nbytes;
                    }
                    packed.push_back(Flat{at, regs[i].len, false, regs[i].tag});
                    at += regs[i].len;
                }
                for (uint32_t k : pc.tensors) {
                    dst[k] = at;
                    packed.push_back(Flat{at, sizes[k], false, kNewTag + k});
                    at += sizes[k];
                }
                if (at > end) return ERR_NOSPACE;                 // ruled out by the check above
                if (at < end) packed.push_back(Flat{at, end - at, true, 0});
                work.splice(begin, end, packed);
            }
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
