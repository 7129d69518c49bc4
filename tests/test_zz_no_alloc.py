"""emb_lookup_noalloc (the entry point for callers that cannot allocate) against emb_lookup.

Two pools of the same geometry over the same table take the same batches, one through each entry
point: outputs, hit flags, cache state and counters must be identical (integer and byte work:
bit-exact).  The second call is smaller than the first, so the fixed work space still holds the
first call's lists when it starts.  The pooled case takes the same path with bags of four."""
import numpy as np
import pytest
import torch

from paper_2605_04450_amd import binding as B
from paper_2605_04450_amd import device as Hn
from paper_2605_04450_amd import synth

pytestmark = pytest.mark.gpu


def two_pools(rows, d, n_pages, frac):
    rng = synth.rng_for(0, 41)
    table = Hn.to_device_table(synth.make_table(rng, rows, d, bf16=True))
    page = 16 * 2 * 1 * d * 2
    mk = lambda: Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, 16, 32, table.view(torch.bfloat16), frac)
    return rng, table, mk(), mk()


@pytest.mark.parametrize("bag", [1, 4])
def test_noalloc_lookup_equals_emb_lookup_on_two_calls_in_a_row(bag):
    rows, d = 20000, 128
    rng, table, ref, pool = two_pools(rows, d, 64, 0.5)  # 64 pages x 32 slots x 0.5: 1024 slots for 20000 rows
    sizes = [8192, 1000 * bag]                           # the second call is smaller than the first
    for n in sizes + [4096, 16384]:
        ids = torch.from_numpy(synth.zipf_ids(rng, rows, 1.0, n)).to(Hn.DEV)
        ids[::97] = rows + 5  # some ids outside the table
        out_a = torch.empty((n // bag, d), dtype=torch.bfloat16, device=Hn.DEV)
        out_b = torch.full_like(out_a, 7.0)
        hit_a = torch.empty(n, dtype=torch.uint8, device=Hn.DEV)
        hit_b = torch.full_like(hit_a, 9)
        assert B.emb_lookup(ref.h, ids, out_a, bag, hit_a) == B.OK, B.last_error()
        assert B.emb_lookup_noalloc(pool.h, ids, out_b, bag, hit_b) == B.OK, B.last_error()
        torch.cuda.synchronize()
        assert torch.equal(hit_a, hit_b), n
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), n
        ta, sa = ref.cache_dump()
        tb, sb = pool.cache_dump()
        assert np.array_equal(ta, tb) and np.array_equal(sa, sb), n
        st_a, st_b = ref.stats(), pool.stats()
        assert st_b.pop("ws_allocs") == 0 and st_a.pop("ws_allocs") > 0  # the library's own count of its allocations
        assert st_a == st_b, (st_a, st_b)
    assert ref.stats()["evicted"] > 0 and ref.stats()["hits"] > 0 and ref.stats()["invalid_ids"] > 0
    ref.close()
    pool.close()


def test_noalloc_lookup_rejects_batches_beyond_its_work_space():
    rows, d = 5000, 512
    rng, table, ref, pool = two_pools(rows, d, 64, 0.5)
    ref.close()
    n = B.NOALLOC_MAX_LOOKUPS + 1
    ids = torch.zeros(n, dtype=torch.int64, device=Hn.DEV)
    out = torch.empty((n, d), dtype=torch.bfloat16, device=Hn.DEV)
    before = pool.stats()
    assert B.emb_lookup_noalloc(pool.h, ids, out, 1, None) == B.ERANGE
    n = B.NOALLOC_MAX_ROW_BYTES_TOTAL // (d * 2) + 1  # fewer lookups, but their rows do not fit
    assert B.emb_lookup_noalloc(pool.h, ids[:n], out[:n], 1, None) == B.ERANGE
    assert "work space" in B.last_error()
    assert pool.stats() == before  # nothing was done, not even the LRU clock moved
    n = B.NOALLOC_MAX_ROW_BYTES_TOTAL // (d * 2)
    assert B.emb_lookup_noalloc(pool.h, ids[:n], out[:n], 1, None) == B.OK
    torch.cuda.synchronize()
    want = table.view(torch.bfloat16)[0].to(Hn.DEV)
    assert torch.equal(out[:n].view(torch.int16), want.view(torch.int16).expand(n, d))
    pool.close()
