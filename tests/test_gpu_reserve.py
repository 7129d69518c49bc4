"""pool_reserve: after it, calls within the reserved sizes allocate nothing (pool_stats.ws_allocs stays
constant) and give the results they gave before."""
import numpy as np
import pytest
import torch

from paper_2605_04450_amd import binding as B
from paper_2605_04450_amd import device as Hn
from paper_2605_04450_amd import synth

pytestmark = pytest.mark.gpu


def test_reserved_work_spaces_are_never_regrown():
    L, d, H, pt, rows = 2, 128, 2, 64, 20000
    rng = synth.rng_for(1, 5)
    table = Hn.to_device_table(synth.make_table(rng, rows, d, bf16=True))
    w = synth.make_weights(rng, L, d, H, 4096, 16, True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, 4096, 16, 4096.0, w)

    def run(pool, reserve):
        if reserve:
            assert B.pool_reserve(pool.h, model.h, max_lookups=40000, max_requests=40, max_new_tokens=40000,
                                  max_seq_tokens=4096) == B.OK, B.last_error()
        base = pool.stats()["ws_allocs"]
        r = np.random.default_rng(9)
        outs = []
        for step in range(6):
            n_req = int(r.integers(1, 40))
            lens = r.integers(1, 4096, size=n_req)
            lens = np.minimum((lens * (r.integers(2000, 40000) / lens.sum())).astype(np.int64) + 1, 4096)
            reqs, n_pt, n_ts, N = synth.make_requests([0] * n_req, lens.tolist(), pt)
            ids = torch.from_numpy(synth.zipf_ids(r, rows, 1.0, N)).to(Hn.DEV)
            x, _ = pool.lookup(ids)
            pts = torch.arange(1024, 1024 + n_pt, dtype=torch.int32, device=Hn.DEV)  # above every EMB page
            ts = torch.from_numpy(np.concatenate([synth.timestamps(r, int(s)) for s in lens])).to(Hn.DEV)
            out = torch.empty_like(x)
            assert B.hstu_step(pool.h, model.h, reqs, pts, x, ts, out) == B.OK, B.last_error()
            outs.append(out)
            assert B.pool_set_split(pool.h, 0.2 + 0.02 * step)[0] == B.OK
        torch.cuda.synchronize()
        return outs, pool.stats()["ws_allocs"] - base

    page = model.page_size()
    n_pages = 2048
    mk = lambda: Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), 0.2)
    grown, reserved = mk(), mk()
    outs_a, allocs_a = run(grown, False)
    outs_b, allocs_b = run(reserved, True)
    assert allocs_a > 0 and allocs_b == 0, (allocs_a, allocs_b)
    for a, b in zip(outs_a, outs_b):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # beyond the reserved sizes a call still works, and grows what it needs
    n = 50000
    ids = torch.from_numpy(synth.zipf_ids(rng, rows, 1.0, n)).to(Hn.DEV)
    before = reserved.stats()["ws_allocs"]
    reserved.lookup(ids)
    assert reserved.stats()["ws_allocs"] > before
    for p in (grown, reserved):
        p.close()
    model.close()
