"""A scaled-down serving loop (the trade-off of the paper's Sec. III: HBM given to the EMB cache saves host
fetches, HBM given to the KV cache saves recomputation) run side by side on the library and on the oracle.

Per batch: a few users are drawn by popularity; a user whose KV is still resident (kv_seq_lookup) computes
only its newest tokens against the cached prefix, any other is reserved afresh (kv_seq_reserve, which may
reclaim cold users' pages) and recomputes its whole history; every new token looks up eight sum-pooled
features; the sequences are pinned while the step runs.  At three splits, with pool_set_split in between.
Page lists, KV hit sets, hit flags, pooled rows and counters must be identical; step outputs must agree
within the floating-point tolerance (each side reads the prefix it cached itself)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_04450_amd import binding as B
from paper_2605_04450_amd import device as Hn
from paper_2605_04450_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

COUNTERS = ("lookups", "hits", "misses", "unique_misses", "inserted", "evicted", "bypassed", "shrink_evicted",
            "shrink_moved", "pages_emb", "pages_kv_free", "pages_kv_used", "seqs_resident", "seqs_evicted", "batch")


def test_serving_loop_follows_the_oracle_at_three_splits():
    L, d, H, pt, bag, new = 2, 128, 2, 16, 8, 32
    rows, users, n_pages = 16000, 48, 512
    rng = synth.rng_for(5, 3)
    table = synth.make_table(rng, rows, d, bf16=True)
    w = synth.make_weights(rng, L, d, H, 1024, 16, True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, 1024, 16, 1024.0, w)
    page = model.page_size()
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, Hn.to_device_table(table), 0.7)
    orc = oracle.Pool(n_pages, pt, page // (d * 2), 32, 0.7)
    cfg = oracle.make_cfg(L, d, H, pt, 1024, 16, 1024.0, 1e-6, True)
    okv = np.zeros(n_pages * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    lens = synth.history_lengths(rng, users, 300, 64, 900)
    ts_user = [synth.timestamps(rng, int(s)) for s in lens]
    pop = np.arange(1, users + 1, dtype=np.float64) ** -0.8
    pop /= pop.sum()
    kv_hits = kv_misses = reclaimed = 0
    worst = 0.0
    for phase, frac in enumerate((0.7, 0.3, 0.5)):
        assert B.pool_set_split(pool.h, frac) == orc.set_split(frac)
        for batch in range(17):
            picked = np.unique(rng.choice(users, size=6, p=pop))
            reqs, pages, ts, keys = [], [], [], []
            pto = tso = xo = 0
            for u in picked:
                S = int(lens[u])
                rc_g, tok_g, pg_g = B.kv_seq_lookup(pool.h, int(u))
                rc_o, tok_o, pg_o = orc.kv_lookup(int(u))
                assert (rc_g, tok_g) == (rc_o, tok_o), (phase, batch, u)
                if rc_g == B.OK and tok_g == S:      # KV hit: only the newest tokens
                    assert np.array_equal(pg_g, pg_o)
                    P, T, pg = S - new, new, pg_g
                    kv_hits += 1
                else:                                 # miss: reserve (may reclaim cold users), recompute everything
                    before = pool.stats()["seqs_evicted"]
                    rc_g, pg_g = B.kv_seq_reserve(pool.h, int(u), S)
                    rc_o, pg_o = orc.kv_reserve(int(u), S)
                    assert rc_g == rc_o, (phase, batch, u, rc_g, rc_o)
                    if rc_g != B.OK:
                        continue                      # no room even after reclaiming: the request is dropped on both sides
                    assert np.array_equal(pg_g, pg_o), (phase, batch, u)
                    reclaimed += pool.stats()["seqs_evicted"] - before
                    P, T, pg = 0, S, pg_g
                    kv_misses += 1
                assert B.kv_seq_pin(pool.h, int(u)) == B.OK and orc.kv_pin(int(u)) == oracle.OK
                keys.append(int(u))
                reqs.append((P, T, pto, tso, xo))
                pages.append(pg)
                ts.append(ts_user[u])
                pto, tso, xo = pto + len(pg), tso + S, xo + T
            if not reqs:
                continue
            N = xo
            ids = synth.multi_feature_ids(rng, rows, bag, 0.9, N)
            x, hit = pool.lookup(torch.from_numpy(ids).to(Hn.DEV), bag)
            rc, ox, ohit = orc.emb_lookup(ids, table, bag)
            assert np.array_equal(hit.cpu().numpy(), ohit), (phase, batch)
            assert np.array_equal(Hn.out_to_numpy(x, B.ELEM_BF16), ox), (phase, batch)
            pts = np.concatenate(pages).astype(np.int32)
            tsa = np.concatenate(ts)
            out = torch.empty_like(x)
            rc = B.hstu_step(pool.h, model.h, reqs, torch.from_numpy(pts).to(Hn.DEV), x, torch.from_numpy(tsa).to(Hn.DEV), out)
            assert rc == B.OK, B.last_error()
            rc, ref = oracle.hstu_step(cfg, w, reqs, pts, okv, synth.from_bf16_bits(ox), tsa)
            assert rc == oracle.OK
            torch.cuda.synchronize()
            er, ee = parity.assert_close(out.float().cpu().numpy(), ref, True, "serving loop, split %g, batch %d" % (frac, batch))
            worst = max(worst, er)
            for u in keys:
                assert B.kv_seq_unpin(pool.h, u) == B.OK and orc.kv_unpin(u) == oracle.OK
            st, so = pool.stats(), orc.stats()
            for k in COUNTERS:
                assert st[k] == so[k], (phase, batch, k, st[k], so[k])
        tags, stamps = pool.cache_dump()
        od = orc.dump()
        assert np.array_equal(tags, od["tags"]) and np.array_equal(stamps, od["stamps"]), phase
        assert np.array_equal(B.pool_dump(pool.h)["owner"], od["owner"]), phase
    # the loop really exercised all three outcomes
    assert kv_hits > 10 and kv_misses > 10 and reclaimed > 0, (kv_hits, kv_misses, reclaimed)
    assert pool.stats()["bad_pages"] == 0 and pool.stats()["evicted"] > 0
    model.close()
    pool.close()
