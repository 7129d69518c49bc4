"""Pins for the oracle's pool / KV / EMB-cache simulator (CPU only).

Each test compares the oracle with something other than itself: numbers the
paper prints (tests/golden/paper_closed_forms.txt), textbook LRU and
direct-mapped caches, set-membership brute force, an independently structured
Python model, and conservation invariants.
"""
import collections
import os

import numpy as np
import pytest

import oracle
from paper_2605_04450_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_closed_forms.txt")


def golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def small_table(rows=4096, d=8, seed=1):
    return np.random.default_rng(seed).standard_normal((rows, d)).astype(np.float32)


# --------------------------------------------------------------------------- geometry
def test_geometry_matches_config_sizes():
    # Tiny config: 512 pages of 8 KiB, 256 B rows -> 32 slots/page; half the pool = 8k slots
    p = oracle.Pool(512, 16, 32, 32, 0.5)
    assert p.num_sets == 512 and p.ways(0) == 16 and p.ways(511) == 16
    assert p.stats()["pages_emb"] * 32 == 8192  # "hot cache 8k slots"
    # Mid config: 64 GiB of 256 KiB pages, 512 B rows -> 512 slots/page
    n_pages = (64 << 30) // (256 << 10)
    assert n_pages == 262144
    assert n_pages * 512 // 32 == 4194304


def test_slot_map_is_a_bijection_onto_emb_pages():
    for frac in (0.1, 0.37, 0.5, 0.9):
        p = oracle.Pool(64, 4, 8, 16, frac)
        d = p.dump()
        slots = set()
        for s in range(p.num_sets):
            for w in range(p.ways(s)):
                sl = p.slot_of(s, w)
                assert sl >= 0 and d["owner"][sl // 8] == 1
                slots.add(sl)
            assert p.slot_of(s, p.ways(s)) == -1
        assert len(slots) == p.stats()["pages_emb"] * 8


def test_ways_differ_by_at_most_one_and_sum_to_capacity():
    p = oracle.Pool(64, 4, 8, 16, 0.3)  # 19 pages, G = 4 -> 4 full layers + 3 pages
    w = [p.ways(s) for s in range(p.num_sets)]
    assert set(w) == {4, 5} and sum(w) == 19 * 8
    assert w == sorted(w, reverse=True)  # the extra way goes to the lowest sets


def test_hash_matches_big_integer_arithmetic():
    p = oracle.Pool(96, 4, 8, 32, 0.5)
    S = p.num_sets
    for id_ in [0, 1, 2, 12345, 2**31 - 1, 2**32 - 2, 99999989]:
        assert p.set_of(id_) == (((id_ * 0x9E3779B97F4A7C15) % 2**64) >> 32) % S


# --------------------------------------------------------------------------- paper's numbers
def test_split_change_moves_the_papers_byte_counts():
    g = golden()
    page = 256 << 10
    n_pages = int(g["gpu_hbm_gb"]) * (1 << 30) // page  # the paper's 80 GB part, in GiB pages
    p = oracle.Pool(n_pages, 64, 512, 32, 0.5)
    before = p.stats()["pages_emb"]
    rc, ach = p.set_split(0.5 + g["small_step"])
    assert rc == oracle.OK
    moved = (p.stats()["pages_emb"] - before) * page / (1 << 30)
    assert abs(moved - g["small_step_gb"]) < 1e-3  # 4 % of 80 GB = 3.2 GB
    rc, ach = p.set_split(0.5 + g["small_step"] + g["large_step"])
    moved2 = (p.stats()["pages_emb"] - before) * page / (1 << 30) - moved
    assert abs(moved2 - g["large_step_gb"]) < 1e-3  # 10 % = 8 GB


def test_alpha_domain_is_the_papers():
    g = golden()
    p = oracle.Pool(64, 4, 8, 32, 0.5)
    for bad in (g["alpha_min"] - 0.01, g["alpha_max"] + 0.01, -1.0, float("nan")):
        assert p.set_split(bad)[0] == oracle.EINVAL
    step = g["alpha_step"]
    a = g["alpha_min"]
    while a <= g["alpha_max"] + 1e-9:  # every point of the action grid is accepted
        rc, ach = p.set_split(round(a, 10))
        assert rc == oracle.OK
        assert p.stats()["pages_emb"] == int(np.floor(round(a, 10) * 64 + 0.5))
        a += step


# --------------------------------------------------------------------------- KV side
def conservation(p):
    st = p.stats()
    d = p.dump()
    assert st["pages_emb"] + st["pages_kv_used"] + st["pages_kv_free"] == st["pages_total"]
    assert (d["owner"] == 1).sum() == st["pages_emb"]
    assert (d["owner"] == 0).sum() == st["pages_kv_free"]
    assert sorted(d["emb_pages"].tolist()) == np.nonzero(d["owner"] == 1)[0].tolist()


def test_kv_pages_lowest_first_and_never_move():
    p = oracle.Pool(64, 4, 8, 32, 0.25)  # pages 0..15 EMB
    rc, a = p.kv_reserve(7, 10)  # 3 pages
    assert rc == oracle.OK and a.tolist() == [16, 17, 18]
    rc, b = p.kv_reserve(9, 4)
    assert b.tolist() == [19]
    rc, a2 = p.kv_reserve(7, 17)  # grows to 5 pages, old pages keep their place
    assert a2.tolist() == [16, 17, 18, 20, 21]
    for frac in (0.5, 0.3, 0.7, 0.1, 0.6):
        p.set_split(frac)
        conservation(p)
        assert p.kv_lookup(7)[2].tolist() == [16, 17, 18, 20, 21]
        assert p.kv_lookup(9)[2].tolist() == [19]
    assert p.kv_lookup(7)[1] == 17


def test_growth_reclaims_cold_unpinned_sequences_in_lru_order_then_defers():
    p = oracle.Pool(32, 4, 8, 32, 0.25)  # 8 EMB pages, 24 KV pages
    for key in (1, 2, 3, 4):
        assert p.kv_reserve(key, 24)[0] == oracle.OK  # 6 pages each: KV side full
    assert p.stats()["pages_kv_free"] == 0
    p.kv_pin(2)       # in flight
    p.kv_pin(1)
    p.kv_unpin(1)     # touched most recently, but not pinned
    rc, ach = p.set_split(0.5)  # needs 8 pages -> evicts 3 then 4 (oldest stamps)
    assert rc == oracle.OK and ach == 0.5
    assert p.kv_lookup(3)[0] == oracle.NOT_FOUND and p.kv_lookup(4)[0] == oracle.NOT_FOUND
    assert p.kv_lookup(1)[0] == oracle.OK and p.kv_lookup(2)[0] == oracle.OK
    conservation(p)
    rc, ach = p.set_split(0.9)  # needs 13 more; only seq 1 (6) + 4 free are reclaimable
    assert rc == oracle.DEFERRED and ach < 0.9
    assert p.kv_lookup(2)[0] == oracle.OK  # pinned blocks are never evicted
    assert p.kv_lookup(1)[0] == oracle.NOT_FOUND
    assert p.stats()["pages_emb"] == 16 + 10
    conservation(p)
    assert p.stats()["seqs_evicted"] == 3


def test_reserve_fails_cleanly_when_everything_is_pinned():
    p = oracle.Pool(32, 4, 8, 32, 0.5)
    assert p.kv_reserve(1, 40)[0] == oracle.OK  # 10 pages
    p.kv_pin(1)
    before = p.stats()
    assert p.kv_reserve(2, 40)[0] == oracle.ENOMEM  # only 6 free, seq 1 pinned
    assert p.stats() == before
    assert p.kv_release(1) == oracle.EBUSY
    p.kv_unpin(1)
    assert p.kv_reserve(2, 40)[0] == oracle.OK  # now evicts seq 1
    assert p.kv_lookup(1)[0] == oracle.NOT_FOUND


# --------------------------------------------------------------------------- EMB cache
def test_one_set_single_id_batches_is_textbook_lru():
    # 32 pages, 1 slot each, 32 ways -> one set; alpha = 0.25 -> 8 ways, fully associative
    p = oracle.Pool(32, 4, 1, 32, 0.25)
    assert p.num_sets == 1 and p.ways(0) == 8
    tab = small_table(64)
    rng = np.random.default_rng(3)
    lru = collections.OrderedDict()
    for step in range(3000):
        id_ = int(rng.integers(0, 20)) if rng.random() < 0.8 else int(rng.integers(0, 64))
        rc, out, hit = p.emb_lookup([id_], tab)
        expect = id_ in lru
        if expect:
            lru.move_to_end(id_)
        else:
            if len(lru) == 8:
                lru.popitem(last=False)
            lru[id_] = True
        assert bool(hit[0]) == expect, step
        assert np.array_equal(out[0], tab[id_])
    st = p.stats()
    assert st["hits"] + st["misses"] == st["lookups"] == 3000
    assert set(p.dump()["tags"][0][:8].tolist()) == set(lru.keys())


def test_one_way_is_a_direct_mapped_cache():
    p = oracle.Pool(8, 4, 16, 1, 1.0)  # w_max = 1, whole pool EMB: 128 sets x 1 way
    assert p.num_sets == 128 and p.ways(5) == 1
    tab = small_table(4096)
    rng = np.random.default_rng(4)
    last = {}
    for step in range(4000):
        id_ = int(rng.integers(0, 600))
        s = p.set_of(id_)
        rc, out, hit = p.emb_lookup([id_], tab)
        assert bool(hit[0]) == (last.get(s) == id_)
        last[s] = id_


def test_large_cache_hit_iff_seen_in_an_earlier_batch():
    p = oracle.Pool(512, 16, 32, 32, 0.5)
    tab = small_table(100000, 4)
    rng = synth.rng_for(1)
    seen = set()
    for b in range(6):
        ids = synth.zipf_ids(rng, 100000, 1.0, 700)
        rc, out, hit = p.emb_lookup(ids, tab)
        assert np.array_equal(out, tab[ids])  # gathered rows equal table rows
        assert hit.tolist() == [int(i in seen) for i in ids.tolist()]
        seen.update(ids.tolist())
    st = p.stats()
    assert st["evicted"] == 0 and st["bypassed"] == 0  # premise of the test
    assert st["hits"] + st["misses"] == st["lookups"] == 4200
    assert st["unique_misses"] == st["inserted"] == len(seen)
    tags = p.dump()["tags"]
    assert set(tags[tags != oracle.TAG_EMPTY].tolist()) == seen


class PyCache:
    """Independent model: per set a dict id -> [last batch, arrival order], no way arrays.
    Victim order among equal stamps follows way order, which for a set that has never
    shrunk is the order in which ways were first filled and later overwritten in place."""

    def __init__(self, n_sets, ways_fn, set_fn):
        self.sets = [[] for _ in range(n_sets)]  # list index = way
        self.ways_fn, self.set_fn, self.t = ways_fn, set_fn, 0

    def lookup(self, ids):
        self.t += 1
        hits = []
        for i in ids:
            ent = [e for e in self.sets[self.set_fn(i)] if e is not None and e[0] == i]
            hits.append(1 if ent else 0)
        for i, h in zip(ids, hits):
            if h:
                for e in self.sets[self.set_fn(i)]:
                    if e is not None and e[0] == i:
                        e[1] = self.t
        done = set()
        for i, h in zip(ids, hits):
            if h or i in done:
                continue
            done.add(i)
            s = self.set_fn(i)
            ways = self.sets[s]
            nw = self.ways_fn(s)
            while len(ways) < nw:
                ways.append(None)
            free = [w for w in range(nw) if ways[w] is None]
            if free:
                ways[free[0]] = [i, self.t]
                continue
            cand = sorted((ways[w][1], w) for w in range(nw) if ways[w][1] < self.t)
            if cand:
                ways[cand[0][1]] = [i, self.t]
        return hits


@pytest.mark.parametrize("n_pages,spp,w_max,frac,alphabet,batch", [
    (32, 1, 32, 0.25, 24, 7),     # one set, 8 ways, heavy pressure, bypasses happen
    (32, 2, 16, 0.5, 60, 16),     # 4 sets x 8 ways
    (64, 8, 16, 0.3, 900, 64),    # uneven ways (4 or 5)
    (16, 4, 2, 0.5, 200, 33),     # 32 sets x 1 way
])
def test_batches_against_independent_python_model(n_pages, spp, w_max, frac, alphabet, batch):
    p = oracle.Pool(n_pages, 4, spp, w_max, frac)
    model = PyCache(p.num_sets, p.ways, p.set_of)
    tab = small_table(alphabet, 4)
    rng = np.random.default_rng(n_pages + alphabet)
    for b in range(60):
        ids = rng.integers(0, alphabet, size=batch)
        rc, out, hit = p.emb_lookup(ids, tab)
        assert hit.tolist() == model.lookup(ids.tolist()), b
        d = p.dump()
        for s in range(p.num_sets):
            got = [(int(t), int(st)) for t, st in zip(d["tags"][s], d["stamps"][s]) if t != oracle.TAG_EMPTY]
            want = [(e[0], e[1]) for e in model.sets[s] if e is not None]
            assert got == want, (b, s)
    st = p.stats()
    assert st["hits"] + st["misses"] == st["lookups"]
    assert st["inserted"] + st["bypassed"] == st["unique_misses"]


def test_duplicates_of_a_missing_id_all_miss_and_insert_once():
    p = oracle.Pool(32, 4, 2, 16, 0.5)
    tab = small_table(100, 4)
    rc, out, hit = p.emb_lookup([5, 5, 9, 5, 9], tab)
    assert hit.tolist() == [0, 0, 0, 0, 0]
    st = p.stats()
    assert (st["misses"], st["unique_misses"], st["inserted"]) == (5, 2, 2)
    rc, out, hit = p.emb_lookup([9, 5, 7], tab)
    assert hit.tolist() == [1, 1, 0]


def test_permuting_a_batch_permutes_flags_and_keeps_the_resident_set():
    tab = small_table(5000, 4)
    rng = np.random.default_rng(11)
    batches = [rng.integers(0, 5000, size=300) for _ in range(5)]
    perm = [rng.permutation(300) for _ in range(5)]
    a = oracle.Pool(512, 16, 32, 32, 0.5)
    b = oracle.Pool(512, 16, 32, 32, 0.5)
    for ids, pm in zip(batches, perm):
        _, _, ha = a.emb_lookup(ids, tab)
        _, _, hb = b.emb_lookup(ids[pm], tab)
        assert np.array_equal(ha[pm], hb)
    assert a.stats()["evicted"] == 0
    da, db = a.dump(), b.dump()
    for s in range(a.num_sets):  # same resident ids and stamps; ways may differ
        assert sorted(zip(da["tags"][s], da["stamps"][s])) == sorted(zip(db["tags"][s], db["stamps"][s]))


def test_invalid_ids_are_counted_and_zero_filled():
    p = oracle.Pool(32, 4, 2, 16, 0.5)
    tab = small_table(100, 4)
    rc, out, hit = p.emb_lookup([3, -1, 100, 99], tab)
    assert hit.tolist() == [0, 0, 0, 0]
    assert np.array_equal(out[0], tab[3]) and np.array_equal(out[3], tab[99])
    assert not out[1].any() and not out[2].any()
    st = p.stats()
    assert st["invalid_ids"] == 2 and st["lookups"] == 2


def test_pooled_rows_are_fp32_left_to_right_sums_rounded_once():
    rng = np.random.default_rng(5)
    tab32 = (rng.standard_normal((500, 8)) * 100).astype(np.float32)
    p = oracle.Pool(32, 4, 2, 16, 0.5)
    ids = rng.integers(0, 500, size=8 * 40)
    rc, out, hit = p.emb_lookup(ids, tab32, bag=8)
    want = tab32[ids].reshape(40, 8, 8)
    acc = want[:, 0, :].copy()
    for f in range(1, 8):
        acc = (acc + want[:, f, :]).astype(np.float32)  # numpy fp32 adds are IEEE, in order
    assert np.array_equal(out, acc)
    # bf16 storage: same sum in fp32, one rounding; compare with torch's bf16 conversion
    import torch
    tabb = synth.to_bf16_bits(tab32)
    q = oracle.Pool(32, 4, 2, 16, 0.5)
    rc, outb, _ = q.emb_lookup(ids, tabb, bag=8)
    vals = synth.from_bf16_bits(tabb)[ids].reshape(40, 8, 8)
    acc = vals[:, 0, :].copy()
    for f in range(1, 8):
        acc = (acc + vals[:, f, :]).astype(np.float32)
    want_bits = torch.from_numpy(acc).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(outb, want_bits)
    assert len(hit) == 320 and q.stats()["lookups"] == 320


def test_shrink_keeps_most_recent_entries_and_moves_only_displaced_ones():
    p = oracle.Pool(32, 4, 2, 16, 0.75)  # G = 2, 4 sets, 12 ways each
    tab = small_table(2000, 4)
    rng = np.random.default_rng(8)
    for b in range(12):
        p.emb_lookup(rng.integers(0, 2000, size=12), tab)
    before = p.dump()
    ways_before = [p.ways(s) for s in range(4)]
    rc, ach = p.set_split(0.40625)  # 13 pages: 6 full layers + 1 page -> sets 0,1 get 7 ways
    assert rc == oracle.OK
    ways_after = [p.ways(s) for s in range(4)]
    assert ways_after == [7, 7, 6, 6]
    after = p.dump()
    moved = 0
    for s in range(4):
        ent = [(int(before["stamps"][s][w]), w, int(before["tags"][s][w]))
               for w in range(ways_before[s]) if before["tags"][s][w] != oracle.TAG_EMPTY]
        b_ = ways_after[s]
        # victims leave in ascending (stamp, way) order, exactly as on insertion,
        # so the survivors are the b entries with the greatest (stamp, way)
        keep = sorted(ent, key=lambda e: (e[0], e[1]), reverse=True)[:b_]
        keep_ids = {e[2] for e in keep}
        got = {int(t) for t in after["tags"][s][:b_] if t != oracle.TAG_EMPTY}
        assert got == keep_ids
        assert (after["tags"][s][b_:] == oracle.TAG_EMPTY).all()
        for st_, w, tg in keep:  # entries below the new way count stay where they were
            if w < b_:
                assert after["tags"][s][w] == tg and after["stamps"][s][w] == st_
            else:
                moved += 1
        movers = [e for e in sorted(keep, key=lambda e: e[1]) if e[1] >= b_]
        holes = [w for w in range(b_) if before["tags"][s][w] == oracle.TAG_EMPTY
                 or int(before["tags"][s][w]) not in keep_ids]
        for (st_, w, tg), h in zip(movers, holes):  # in way order into ascending holes
            assert after["tags"][s][h] == tg and after["stamps"][s][h] == st_
    assert p.stats()["shrink_moved"] == moved
    conservation(p)
    # growing again exposes empty ways only; nothing resident is lost
    p.set_split(0.75)
    again = p.dump()
    for s in range(4):
        assert np.array_equal(again["tags"][s], after["tags"][s])


def test_outputs_do_not_depend_on_the_split():
    tab = small_table(3000, 4)
    rng = np.random.default_rng(2)
    batches = [rng.integers(0, 3000, size=200) for _ in range(6)]
    outs = []
    for frac in (0.1, 0.5, 0.9):
        p = oracle.Pool(64, 4, 4, 32, frac)
        outs.append([p.emb_lookup(b, tab)[1] for b in batches])
    for k in range(6):
        assert np.array_equal(outs[0][k], outs[1][k]) and np.array_equal(outs[1][k], outs[2][k])


def test_zipf_hit_rate_is_in_the_harmonic_ballpark():
    # sanity, not parity: an LRU cache of C slots on Zipf(1.0) over N rows hits
    # roughly H_C / H_N of the time once warm
    N, C = 100000, 8192
    p = oracle.Pool(512, 16, 32, 32, 0.5)
    tab = small_table(N, 4)
    rng = synth.rng_for(1, 5)
    for b in range(40):
        p.emb_lookup(synth.zipf_ids(rng, N, 1.0, 1024), tab, want_out=False)
    s0 = p.stats()
    for b in range(40):
        p.emb_lookup(synth.zipf_ids(rng, N, 1.0, 1024), tab, want_out=False)
    s1 = p.stats()
    rate = (s1["hits"] - s0["hits"]) / (s1["lookups"] - s0["lookups"])
    h = lambda n: np.log(n) + 0.5772
    assert 0.6 * h(C) / h(N) < rate < 1.15 * h(C) / h(N)


# --------------------------------------------------------------------------- refill of empty ways
def test_refill_of_an_empty_cache_leaves_what_the_same_lookups_would_leave():
    # with room for every id, "lowest empty way in order of first occurrence" is also what a lookup batch does
    ids = np.random.default_rng(3).permutation(3000)[:900].tolist() + [7, 7, 11]
    a, b = oracle.Pool(512, 16, 32, 32, 0.5), oracle.Pool(512, 16, 32, 32, 0.5)
    rc, n_ins = a.emb_refill(ids, 100000)
    b.emb_lookup(ids, (100000, 4, np.float32), want_out=False)
    assert rc == 0 and n_ins == len(set(ids)) == b.stats()["inserted"]
    da, db = a.dump(), b.dump()
    assert np.array_equal(da["tags"], db["tags"]) and np.array_equal(da["stamps"], db["stamps"])
    sa = a.stats()
    assert (sa["lookups"], sa["hits"], sa["misses"], sa["unique_misses"], sa["evicted"], sa["bypassed"]) == (0,) * 6
    assert sa["inserted"] == n_ins and sa["batch"] == 1  # a refill is a batch of its own in LRU time


def test_refill_never_evicts_and_fills_min_of_new_ids_and_empty_ways_per_set():
    p = oracle.Pool(32, 4, 2, 16, 0.5)  # 4 sets x 8 ways
    rng = np.random.default_rng(8)
    p.emb_lookup(rng.integers(0, 40, size=30), (4000, 4, np.float32), want_out=False)
    before = p.dump()
    resident = {s: [int(t) for t in before["tags"][s] if t != oracle.TAG_EMPTY] for s in range(p.num_sets)}
    ids = rng.permutation(np.arange(1000, 1100)).tolist() + [-4, 4000, 5]  # new ids, two invalid, maybe one resident
    rc, n_ins = p.emb_refill(ids, 4000)
    after = p.dump()
    expect = 0
    for s in range(p.num_sets):
        kept = before["tags"][s] != oracle.TAG_EMPTY
        assert np.array_equal(after["tags"][s][kept], before["tags"][s][kept])      # nobody left, nobody moved
        assert np.array_equal(after["stamps"][s][kept], before["stamps"][s][kept])  # and nobody was touched
        new_here = []
        for i in ids:
            if 0 <= i < 4000 and p.set_of(i) == s and i not in resident[s] and i not in new_here:
                new_here.append(i)
        room = p.ways(s) - len(resident[s])
        got = [int(t) for t, k in zip(after["tags"][s], kept) if not k and t != oracle.TAG_EMPTY]
        assert got == new_here[:room]  # first come first served, lowest empty way first
        expect += min(len(new_here), room)
    assert n_ins == expect and p.stats()["evicted"] == 0


def test_refilled_rows_age_between_the_batches_around_them():
    # one set of 4 ways: A enters in batch 1, B and C by a refill (batch 2), D in batch 3 -> full.
    # Batch 4 brings two new ids: the victims are A (oldest), then B (refilled, lower way than C).
    p = oracle.Pool(32, 1, 1, 32, 0.125)
    assert p.num_sets == 1 and p.ways(0) == 4
    tab = (1000, 4, np.float32)
    p.emb_lookup([10], tab, want_out=False)
    assert p.emb_refill([20, 30], 1000) == (0, 2)
    p.emb_lookup([40], tab, want_out=False)
    assert p.dump()["tags"][0][:4].tolist() == [10, 20, 30, 40]
    assert p.dump()["stamps"][0][:4].tolist() == [1, 2, 2, 3]
    rc, _, hit = p.emb_lookup([20, 50, 60], tab, want_out=False)  # 20 is resident thanks to the refill
    assert hit.tolist() == [1, 0, 0]
    assert p.dump()["tags"][0][:4].tolist() == [50, 20, 60, 40]  # 10 left first, then 30 (20 was just used)
    assert p.emb_refill([70], 1000) == (0, 0)  # a full set takes nothing


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_refill_against_a_dictionary_model_on_tiny_caches(seed):
    rng = np.random.default_rng(100 + seed)
    p = oracle.Pool(16, 4, 2, 4, 0.5)  # 4 sets x 2 ways
    model = {s: [] for s in range(p.num_sets)}  # resident ids per set in way order (no holes: nothing shrinks here)
    for step in range(40):
        ids = rng.integers(-2, 64, size=int(rng.integers(0, 12))).tolist()
        want = 0
        for i in ids:
            if not 0 <= i < 60:
                continue
            s = p.set_of(i)
            if i not in model[s] and len(model[s]) < p.ways(s):
                model[s].append(i)
                want += 1
        rc, n_ins = p.emb_refill(ids, 60)
        assert (rc, n_ins) == (0, want), step
        tags = p.dump()["tags"]
        for s in range(p.num_sets):
            assert [int(t) for t in tags[s] if t != oracle.TAG_EMPTY] == model[s], (step, s)
