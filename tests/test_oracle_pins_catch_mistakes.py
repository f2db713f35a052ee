"""Do the oracle's pins have teeth?  (CPU only.)

Every pin in test_oracle_*.py compares the oracle with something outside it:
published vectors, values computed when the build was specified, closed
forms, layouts worked out by hand.  Here plausible mistakes are planted -- in
a deliberately parametrised copy of the fingerprint, and in the oracle's own
Reuse Store by swapping one of its functions for a wrong one -- and each must
be caught by at least one of those pins.  Nothing here defines correctness:
the parametrised copy only manufactures wrong answers.
"""
import os
import struct

import pytest

import oracle.reuse_store as rs
from recipes import build, read_pairs
from test_oracle_fingerprint import GOLD, published

M64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def make_fingerprint(s1=30, s2=27, s3=31, m1=0xBF58476D1CE4E5B9, m2=0x94D049BB133111EB, add_gamma=True,
                     key="xor", first_index=0, step=GAMMA, endian="little", pad=0, reduce="sum",
                     word_bytes=8, final_shift=True):
    def mix(x):
        z = (x + GAMMA) & M64 if add_gamma else x
        z = ((z ^ (z >> s1)) * m1) & M64
        z = ((z ^ (z >> s2)) * m2) & M64
        return z ^ (z >> s3) if final_shift else z

    def fp(data):
        total = 0
        for i in range((len(data) + word_bytes - 1) // word_bytes):
            chunk = data[word_bytes * i:word_bytes * (i + 1)].ljust(word_bytes, bytes([pad]))
            w = int.from_bytes(chunk, endian)
            k = ((first_index + i) * step) & M64
            x = (w ^ k) if key == "xor" else (w + k) & M64 if key == "add" else w
            t = mix(x)
            if key == "after":
                t ^= k
            total = (total + t) & M64 if reduce == "sum" else total ^ t
        return total
    return fp


def external_pins_hold(fp):
    """The pins of test_oracle_fingerprint.py that rest on data from outside
    the oracle, applied to any candidate function."""
    vec = published()
    try:
        acc = 0
        assert fp(b"") == 0
        for w in range(3):
            acc = (acc + vec[(0, w)]) & M64
            assert fp(bytes(8 * (w + 1))) == acc
        words = [((i * GAMMA) & M64) ^ ((1234567 + i * GAMMA) & M64) for i in range(5)]
        assert fp(b"".join(struct.pack("<Q", w) for w in words)) == sum(vec[(1234567, i)] for i in range(5)) & M64
        for n in (1, 2, 7, 64):
            data = b"".join(struct.pack("<Q", ((i * GAMMA) & M64) ^ 1) for i in range(n))
            assert fp(data) == (n * vec[(1, 0)]) & M64
        assert fp(b"\x01" + bytes(7)) == vec[(1, 0)]
        assert fp(b"\x01") == vec[(1, 0)]
        for recipe, val in read_pairs(os.path.join(GOLD, "specified_fingerprints.txt")):
            assert fp(build(recipe)) == val
    except AssertionError:
        return False
    return True


FINGERPRINT_MISTAKES = {
    "first shift 31": dict(s1=31),
    "second shift 26": dict(s2=26),
    "last shift 30": dict(s3=30),
    "multipliers swapped": dict(m1=0x94D049BB133111EB, m2=0xBF58476D1CE4E5B9),
    "state not advanced by gamma": dict(add_gamma=False),
    "last xor-shift dropped": dict(final_shift=False),
    "key added instead of xored": dict(key="add"),
    "no position key": dict(key="none"),
    "key applied after the mix": dict(key="after"),
    "index from 1": dict(first_index=1),
    "key step off by two": dict(step=GAMMA + 2),
    "big-endian words": dict(endian="big"),
    "tail padded with ones": dict(pad=0xFF),
    "xor instead of sum": dict(reduce="xor"),
    "4-byte words": dict(word_bytes=4),
}


def test_the_parametrised_copy_can_be_right():
    assert external_pins_hold(make_fingerprint())


@pytest.mark.parametrize("name", sorted(FINGERPRINT_MISTAKES))
def test_a_wrong_fingerprint_fails_an_external_pin(name):
    assert not external_pins_hold(make_fingerprint(**FINGERPRINT_MISTAKES[name])), name


# ---------------------------------------------------------------- Reuse Store
def first_fit(regions, need, lo=0, hi=None):
    hi = len(regions) if hi is None else hi
    for i in range(lo, hi):
        if regions[i][2] and regions[i][1] >= need:
            return i
    return None


def worst_fit(regions, need, lo=0, hi=None):
    hi = len(regions) if hi is None else hi
    pick = None
    for i in range(lo, hi):
        if regions[i][2] and regions[i][1] >= need and (pick is None or regions[i][1] > regions[pick][1]):
            pick = i
    return pick


def best_fit_highest_offset_on_ties(regions, need, lo=0, hi=None):
    hi = len(regions) if hi is None else hi
    pick = None
    for i in range(lo, hi):
        if regions[i][2] and regions[i][1] >= need and (pick is None or regions[i][1] <= regions[pick][1]):
            pick = i
    return pick


def carve_high_end(regions, i, need, tag=None):
    off, length, _free, _tag = regions[i]
    if length == need:
        regions[i] = [off, need, False, tag]
        return off
    regions[i] = [off, length - need, True, None]
    regions.insert(i + 1, [off + length - need, need, False, tag])
    return off + length - need


def try_packing_accepts_exact_fits(sizes, tensors, c1, c2):
    t1, t2 = [], []
    for k in tensors:
        if sizes[k] > min(c1, c2):
            return [], []
        if c1 >= c2:
            t1.append(k)
            c1 -= sizes[k]
        else:
            t2.append(k)
            c2 -= sizes[k]
    return t1, t2


def try_packing_fills_the_smaller_bin(sizes, tensors, c1, c2):
    t1, t2 = [], []
    for k in tensors:
        if sizes[k] >= min(c1, c2):
            return [], []
        if c1 < c2:
            t1.append(k)
            c1 -= sizes[k]
        else:
            t2.append(k)
            c2 -= sizes[k]
    return t1, t2


def cost_without_alpha(self, e):
    total = 0.0
    for m in e.owners:
        p, b, _a = self.cost_params.get(m, (1.0, 1.0, 1.0))
        total += p * (float(e.nbytes) / b)
    return total


def cost_times_bandwidth(self, e):
    total = 0.0
    for m in e.owners:
        p, b, a = self.cost_params.get(m, (1.0, 1.0, 1.0))
        total += p * (float(e.nbytes) * b) * a
    return total


def capacity_always_free_only(regions, sub, as_printed):
    return 0 if sub is None else rs.free_bytes(regions, sub)


def capacity_always_as_printed(regions, sub, as_printed):
    return 0 if sub is None else rs.free_bytes(regions, sub) + rs.allocated_bytes(regions, sub)


def merge_cost_counts_free_bytes(regions, sub):
    return sum(r[1] for r in regions[sub[0]:sub[1]] if r[2])


def subspace_not_trimmed(regions, lo, hi):
    return (lo, hi) if any(regions[i][2] for i in range(lo, hi)) else None


def stretches_without_walls(regions, movable):
    sub = rs.subspace(regions, 0, len(regions))
    return [sub] if sub is not None else []


def deal_to_the_smallest_room(regions, subs, sizes, order, cap_as_printed):
    room = [rs.capacity(regions, sub, cap_as_printed) for sub in subs]
    subsets = [[] for _ in subs]
    for k in order:
        fits = [i for i in range(len(room)) if sizes[k] <= room[i]]
        if not fits:
            return None
        b = min(fits, key=lambda i: (room[i], i))
        subsets[b].append(k)
        room[b] -= sizes[k]
    return subsets


def try_packing_text_refuses_exact_fits(sizes, tensors, c1, c2):
    bins, room = ([], []), [c1, c2]
    for k in tensors:
        b = 0 if room[0] >= room[1] else 1
        if sizes[k] >= room[b]:
            return [], []
        bins[b].append(k)
        room[b] -= sizes[k]
    return bins


def smallest_gain_first(regions, pairs, sizes, pack=rs.try_packing, cap_as_printed=False):
    """Algorithm 1 with the partition points tried by ascending gain."""
    pending, done = list(pairs), []
    m = sum(rs.allocated_bytes(regions, sub) for sub, _t in pending)
    while pending:
        sub, tensors = pending.pop(0)
        points = sorted((i for i in range(sub[0], sub[1]) if not regions[i][2]),
                        key=lambda i: (regions[i][1], regions[i][0]))
        for p in points:
            p1, p2 = rs.subspace(regions, sub[0], p), rs.subspace(regions, p + 1, sub[1])
            t1, t2 = pack(sizes, tensors, rs.capacity(regions, p1, cap_as_printed), rs.capacity(regions, p2, cap_as_printed))
            if t1 or t2:
                pending += [(p1, t1), (p2, t2)]
                m -= regions[p][1]
                break
        else:
            done.append((sub, tensors))
    return sorted(done, key=lambda st: st[0][0]), m


def match_ignores_the_length(self, nbytes, fp, incoming, confirm):
    best = None
    for e in self.entries:
        if e.fp == fp and (best is None or e.off < best.off):
            best = e
    return best


def match_takes_the_highest_offset(self, nbytes, fp, incoming, confirm):
    best = None
    for e in self.entries:
        if e.fp == fp and e.nbytes == nbytes and (best is None or e.off > best.off):
            best = e
    return best


def match_never_compares_bytes(self, nbytes, fp, incoming, confirm):
    best = None
    for e in self.entries:
        if e.fp == fp and e.nbytes == nbytes and (best is None or e.off < best.off):
            best = e
    return best


def free_without_merging(regions, off):
    for r in regions:
        if r[0] == off and not r[2]:
            r[2], r[3] = True, None
            return
    raise AssertionError("no allocated region at offset %d" % off)


def reuse_size_counts_slots(self, tensors):
    return sum(rs.round_up(n, self.align) for n, fp, _o in tensors if self._match(n, fp, None, False) is not None)


def pins_of(*names):
    """Pin functions by name; a tuple is (name, argument...) for a parametrised pin."""
    import functools
    import test_oracle_next as nxt
    import test_oracle_store as st
    out = []
    for n in names:
        name, args = (n, ()) if isinstance(n, str) else (n[0], n[1:])
        fn = getattr(st, name, None) or getattr(nxt, name)
        out.append(functools.partial(fn, *args) if args else fn)
    return out


STORE_MISTAKES = [
    ("first fit", rs, "best_fit", first_fit, ["test_hand_derived_best_fit_example"]),
    ("worst fit", rs, "best_fit", worst_fit, ["test_hand_derived_best_fit_example"]),
    ("ties to the highest offset", rs, "best_fit", best_fit_highest_offset_on_ties,
     ["test_ties_take_the_lowest_offset_and_equal_sizes_go_in_index_order"]),
    ("slot at the high end of the region", rs, "carve", carve_high_end, ["test_hand_derived_best_fit_example"]),
    ("TryPacking accepts exact fits", rs, "try_packing", try_packing_accepts_exact_fits,
     ["test_try_packing_follows_the_listing"]),
    ("TryPacking fills the smaller bin", rs, "try_packing", try_packing_fills_the_smaller_bin,
     ["test_try_packing_follows_the_listing", "test_hand_derived_merge_plan"]),
    ("Eq. 2 without alpha", rs.ReuseStoreOracle, "eviction_cost", cost_without_alpha,
     ["test_eviction_cost_is_eq_2", "test_hand_derived_eviction_order"]),
    ("Eq. 2 multiplies by the bandwidth", rs.ReuseStoreOracle, "eviction_cost", cost_times_bandwidth,
     ["test_eviction_cost_is_eq_2", "test_hand_derived_eviction_order"]),
    ("capacity never counts allocated bytes", rs, "capacity", capacity_always_free_only,
     [("test_packing_example_of_the_paper", True), "test_capacity_as_printed_can_hand_a_subspace_more_than_it_holds"]),
    ("capacity always counts allocated bytes", rs, "capacity", capacity_always_as_printed,
     [("test_packing_example_of_the_paper", False), "test_capacity_as_printed_can_hand_a_subspace_more_than_it_holds"]),
    ("merge cost M counts the free bytes", rs, "allocated_bytes", merge_cost_counts_free_bytes,
     [("test_packing_example_of_the_paper", False)]),
    ("a subspace keeps its allocated ends", rs, "subspace", subspace_not_trimmed,
     ["test_a_subspace_begins_and_ends_with_a_free_region"]),
    ("running tensors are no walls", rs, "stretches", stretches_without_walls,
     ["test_running_tensors_are_walls", "test_regions_that_cannot_move_cut_the_pool_into_subspaces"]),
    ("tensors dealt to the subspace with the least room", rs, "deal_over_stretches", deal_to_the_smallest_room,
     ["test_regions_that_cannot_move_cut_the_pool_into_subspaces"]),
    ("the text's packing test refuses exact fits", rs, "try_packing_text", try_packing_text_refuses_exact_fits,
     ["test_try_packing_as_the_text_words_it"]),
    ("the match key is the fingerprint alone", rs.ReuseStoreOracle, "_match", match_ignores_the_length,
     ["test_same_bytes_different_length_do_not_match"]),
    ("of several resident copies the highest offset wins", rs.ReuseStoreOracle, "_match", match_takes_the_highest_offset,
     ["test_duplicates_inside_one_model_and_across_models"]),
    ("confirm trusts the fingerprint", rs.ReuseStoreOracle, "_match", match_never_compares_bytes,
     ["test_confirm_demotes_a_constructed_collision"]),
    ("freed regions are not merged with free neighbours", rs, "free_at", free_without_merging,
     ["test_release_keeps_tensors_matchable_until_evicted"]),
    ("the reuse size counts padded slots", rs.ReuseStoreOracle, "reuse_size", reuse_size_counts_slots,
     ["test_reuse_size_counts_resident_bytes"]),
    ("the smallest gain is tried first", rs, "partitioned_gain_packing", smallest_gain_first,
     [("test_packing_example_of_the_paper", False), ("test_packing_example_of_the_paper", True)]),
]


@pytest.mark.parametrize("case", STORE_MISTAKES, ids=[c[0] for c in STORE_MISTAKES])
def test_a_wrong_store_function_fails_a_hand_derived_pin(case, monkeypatch):
    _name, owner, attr, wrong, pin_names = case
    pins = pins_of(*pin_names)
    for pin in pins:
        pin()                                   # green with the oracle as it stands
    original = getattr(owner, attr)
    monkeypatch.setattr(owner, attr, wrong)
    # names the pin modules bound at import time, and the planner's default argument
    import test_oracle_next as nxt
    import test_oracle_store as st
    for mod in (nxt, st):
        if getattr(mod, attr, None) is original:
            monkeypatch.setattr(mod, attr, wrong)
    defaults = rs.partitioned_gain_packing.__defaults__
    if any(d is original for d in defaults):
        monkeypatch.setattr(rs.partitioned_gain_packing, "__defaults__",
                            tuple(wrong if d is original else d for d in defaults))
    caught = 0
    for pin in pins:
        try:
            pin()
        except (AssertionError, pytest.fail.Exception):     # the latter: an expected NoSpace did not come
            caught += 1
        except (rs.NoSpace, KeyError, IndexError, ValueError):
            caught += 1                         # the mistake broke the plan outright
    assert caught == len(pins), "%d of %d pins noticed" % (caught, len(pins))
