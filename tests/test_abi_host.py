"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host bookkeeping (metadata-only pool) agrees with the oracle's pool simulator."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_04450_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "racer_pool.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int32_t|uint64_t|int64_t|double|char\s*\*)\s*\*?\s*([a-z_0-9]+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert len(names) >= 19 and "pool_create" in names and "hstu_step" in names and "emb_lookup" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_geometry_errors():
    bad = [
        dict(nbytes=64 * 1024, page_size=1000, row_bytes=16),        # bytes % page_size
        dict(nbytes=64 * 1024, page_size=1024, row_bytes=24),        # row_bytes % 16
        dict(nbytes=63 * 1024, page_size=1024, row_bytes=16),        # pages % w_max
        dict(nbytes=64 * 1024, page_size=1024, row_bytes=48),        # page_size % row_bytes
        dict(nbytes=64 * 1024, page_size=1024, row_bytes=16, w_max=24),
        dict(nbytes=64 * 1024, page_size=1024, row_bytes=16, emb_frac0=1.5),
    ]
    for kw in bad:
        args = dict(nbytes=0, page_size=0, row_bytes=16, elem=B.ELEM_F32, page_tokens=4, w_max=32, emb_frac0=0.5)
        args.update(kw)
        rc, h = B.pool_create(None, args["nbytes"], args["page_size"], args["row_bytes"], args["elem"],
                              args["page_tokens"], args["w_max"], None, 0, args["emb_frac0"])
        assert rc == B.EINVAL and h is None, kw


def host_pool(n_pages, pt, spp, w_max, frac):
    rc, h = B.pool_create(None, n_pages * spp * 16, spp * 16, 16, B.ELEM_F32, pt, w_max, None, 0, frac)
    assert rc == B.OK
    return h


def same_state(h, o):
    st, so = B.pool_stats(h), o.stats()
    for k in ("pages_total", "pages_emb", "pages_kv_used", "pages_kv_free", "seqs_resident", "seqs_evicted"):
        assert st[k] == so[k], k
    d, do = B.pool_dump(h), o.dump()
    assert np.array_equal(d["emb_pages"], do["emb_pages"])
    assert np.array_equal(d["owner"], do["owner"])


def test_metadata_only_pool_rejects_device_calls():
    h = host_pool(64, 4, 8, 32, 0.5)
    assert B.load().emb_lookup(h, None, 0, 1, None, None, None) == B.EINVAL
    assert B.load().emb_refill(h, None, 0, None) == B.EINVAL
    assert B.load().pool_add_table(h, None, 10, 64, None) == B.EINVAL
    assert B.load().emb_lookup_tables(h, None, None, 0, 1, None, None, None) == B.EINVAL
    assert B.load().emb_cache_dump(h, None, None) == B.EINVAL
    B.pool_destroy(h)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_host_bookkeeping_matches_oracle_on_random_traces(seed):
    rng = np.random.default_rng(seed)
    n_pages, pt, spp, w_max = 96, 4, 8, 32
    h = host_pool(n_pages, pt, spp, w_max, 0.3)
    o = oracle.Pool(n_pages, pt, spp, w_max, 0.3)
    assert B.pool_num_sets(h) == o.num_sets
    pinned = {}
    for step in range(600):
        op = rng.integers(0, 10)
        key = int(rng.integers(0, 12))
        if op <= 3:
            tokens = int(rng.integers(1, 60))
            rc, pages = B.kv_seq_reserve(h, key, tokens)
            rco, pages_o = o.kv_reserve(key, tokens)
            assert rc == rco, (step, rc, rco)
            if rc == B.OK:
                assert np.array_equal(pages, pages_o), step
        elif op == 4:
            assert B.kv_seq_pin(h, key) == o.kv_pin(key)
            rc, tok, pg = B.kv_seq_lookup(h, key)
            if rc == B.OK:
                pinned[key] = pinned.get(key, 0) + 1
        elif op == 5:
            assert B.kv_seq_unpin(h, key) == o.kv_unpin(key)
        elif op == 6:
            assert B.kv_seq_release(h, key) == o.kv_release(key)
        elif op == 7:
            rc, tok, pg = B.kv_seq_lookup(h, key)
            rco, toko, pgo = o.kv_lookup(key)
            assert (rc, tok) == (rco, toko)
            if rc == B.OK:
                assert np.array_equal(pg, pgo)
        else:
            frac = float(rng.choice(np.round(np.arange(0.08, 0.95, 0.02), 2)))
            rc, ach = B.pool_set_split(h, frac, device=False)
            rco, acho = o.set_split(frac)
            assert rc == rco and (rc < 0 or ach == acho), (step, frac, rc, rco, ach, acho)
        same_state(h, o)
        for s in range(0, o.num_sets, 7):
            for w in (0, 3, 9, 31):
                assert B.pool_slot_of(h, s, w) == o.slot_of(s, w)
    B.pool_destroy(h)


def test_alpha_domain_and_deferral():
    h = host_pool(32, 4, 8, 32, 0.25)
    for bad in (0.05, 0.95, float("nan")):
        assert B.pool_set_split(h, bad, device=False)[0] == B.EINVAL
    for key in (1, 2, 3, 4):
        assert B.kv_seq_reserve(h, key, 24)[0] == B.OK
    B.kv_seq_pin(h, 2)
    rc, ach = B.pool_set_split(h, 0.9, device=False)
    assert rc == B.DEFERRED and ach < 0.9
    assert B.kv_seq_lookup(h, 2)[0] == B.OK          # the pinned block survives
    assert B.kv_seq_reserve(h, 9, 4)[0] == B.ENOMEM  # nothing reclaimable is left
    B.pool_destroy(h)
