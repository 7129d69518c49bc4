"""GPU parity at the full sizes of the five workload configurations, in the launch shapes the
benchmark uses.  The integer side (hit flags, tags, stamps, counters) is compared with the
oracle in full; gathered rows and attention outputs are compared on samples the oracle can
compute one by one (whole short requests, windows of query rows of long ones), plus
properties that hold at any size (rows equal table rows, KV pages never move)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_04450_amd import binding as B
from paper_2605_04450_amd import device as Hn
from paper_2605_04450_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


def pinned_bf16_table(rows, d, seed, may_fail=False):
    """Pinned host table filled with the synthetic bf16 pattern; None if may_fail and the host refuses."""
    import gc
    gc.collect()
    empty = getattr(torch._C, "_host_emptyCache", None)  # hand cached pinned blocks of earlier tests back
    if empty is not None:
        empty()
    try:
        t = torch.empty((rows, d), dtype=torch.int16, pin_memory=True)
    except RuntimeError as e:  # the host cannot pin this much
        if may_fail:
            return None
        pytest.skip("cannot pin a %d x %d bf16 table: %s" % (rows, d, e))
    synth.fill_table_bf16_torch(t, seed, Hn.DEV)
    torch.cuda.synchronize()
    return t


def table_rows_np(table_i16, ids):
    return table_i16[torch.from_numpy(np.asarray(ids, dtype=np.int64))].numpy().view(np.uint16)


def check_cache_state(pool, orc, table_i16, sample=3000):
    st, so = pool.stats(), orc.stats()
    for k in ("lookups", "hits", "misses", "unique_misses", "inserted", "evicted", "bypassed", "invalid_ids",
              "shrink_evicted", "shrink_moved", "pages_emb", "pages_kv_free", "batch"):
        assert st[k] == so[k], (k, st[k], so[k])
    tags, stamps = pool.cache_dump()
    od = orc.dump()
    assert np.array_equal(tags, od["tags"])
    assert np.array_equal(stamps, od["stamps"])
    ss, ww = np.nonzero(tags != B.TAG_EMPTY)
    pick = np.random.default_rng(1).integers(0, len(ss), size=min(sample, len(ss)))
    slots = [orc.slot_of(int(s), int(w)) for s, w in zip(ss[pick], ww[pick])]
    rows = pool.slot_rows(slots)
    want = table_rows_np(table_i16, tags[ss[pick], ww[pick]].astype(np.int64))
    assert np.array_equal(rows, want.view(np.uint8).reshape(len(slots), -1))


def test_mid_config_embedding_side_full_size():
    # Mid: table 10M x 256 bf16 pinned, 64 GiB pool of 256 KiB pages at EMB:KV = 0.5, ~131k lookups per batch
    rows, d, pt, L = 10_000_000, 256, 64, 4
    table = pinned_bf16_table(rows, d, synth.SEED_BASE + 1)
    page = pt * 2 * L * d * 2
    n_pages = (64 << 30) // page
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), 0.5)
    orc = oracle.Pool(n_pages, pt, page // (d * 2), 32, 0.5)
    rng = synth.rng_for(1, 7)
    n = 131440
    hits = []
    for b in range(5):
        ids = synth.zipf_ids(rng, rows, 1.0, n)
        out, hit = pool.lookup(torch.from_numpy(ids).to(Hn.DEV))
        rc, _, ohit = orc.emb_lookup(ids, _rows_only(rows, d), want_out=False)
        assert np.array_equal(hit.cpu().numpy(), ohit), b
        pick = rng.integers(0, n, size=4000)
        got = out[torch.from_numpy(pick).to(Hn.DEV)].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, table_rows_np(table, ids[pick])), b  # gathered rows equal table rows
        hits.append(int(ohit.sum()))
    assert hits[-1] > hits[0]
    check_cache_state(pool, orc, table)
    pool.close()


def _rows_only(rows, d):
    """Shape of a bf16 table for oracle calls that produce no output rows (they read no table data)."""
    return (rows, d, np.uint16)


def test_emb_heavy_config_pooled_lookups_full_size():
    # EMB-heavy: table 100M x 128 bf16 pinned (8 features in disjoint ranges), 50 GiB pool at 0.8,
    # batch 256 x 1024 tokens x 8 features sum-pooled, Zipf(0.8)
    rows, d, pt, L, bag = 100_000_000, 128, 64, 4, 8
    table = pinned_bf16_table(rows, d, synth.SEED_BASE + 3)
    page = pt * 2 * L * d * 2
    n_pages = (50 << 30) // page
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), 0.8)
    orc = oracle.Pool(n_pages, pt, page // (d * 2), 32, 0.8)
    rng = synth.rng_for(3, 7)
    tokens = 256 * 1024
    for b in range(3):
        ids = synth.multi_feature_ids(rng, rows, bag, 0.8, tokens)
        out, hit = pool.lookup(torch.from_numpy(ids).to(Hn.DEV), bag)
        rc, _, ohit = orc.emb_lookup(ids, _rows_only(rows, d), bag, want_out=False)
        assert np.array_equal(hit.cpu().numpy(), ohit), b
        # pooled rows on a sample: fp32 left-to-right sum of the 8 table rows, rounded once (oracle, small table)
        pick = rng.integers(0, tokens, size=1500)
        sub_ids = ids.reshape(tokens, bag)[pick].reshape(-1)
        uniq, inv = np.unique(sub_ids, return_inverse=True)
        sub_table = table_rows_np(table, uniq)
        small = oracle.Pool(64, pt, 32, 32, 0.5)
        rc, want, _ = small.emb_lookup(inv.astype(np.int64), np.ascontiguousarray(sub_table), bag)
        got = out[torch.from_numpy(pick).to(Hn.DEV)].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want), b
    check_cache_state(pool, orc, table)
    pool.close()


def test_long_history_config_attention_on_cached_prefix():
    # Long history: 8 layers, d = 512, 8 heads, bf16; 32 requests with a 16k-token cached prefix (synthetic
    # K,V written straight into shuffled pages) and 512 new tokens scored causally against it
    L, d, H, pt, P, T, Bq = 8, 512, 8, 64, 16384, 512, 32
    n_pos, n_time, n_scale = 16896, 32, 16896.0
    rng = synth.rng_for(2)
    w = synth.make_weights(rng, L, d, H, n_pos, n_time, True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, n_time, n_scale, w)
    page = model.page_size()
    pages_per_req = (P + T + pt - 1) // pt
    n_pages = ((Bq * pages_per_req * 4 // 3) // 32 + 1) * 32
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, None, 0.25)
    first_kv = n_pages // 4
    perm = first_kv + rng.permutation(n_pages - first_kv)
    reqs, n_pt, n_ts, N = synth.make_requests([P] * Bq, [T] * Bq, pt)
    pts = perm[:n_pt].astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng, P + T) for _ in range(Bq)])
    layer = 3
    # synthetic cache: K ~ N(0, d_h^-1/2), V ~ N(0,1), generated on the device per request
    mem = pool.mem.view(torch.bfloat16)
    gen = torch.Generator(device=Hn.DEV)
    gen.manual_seed(1234)
    kv_host = {}
    for r in range(Bq):
        k = (torch.randn((P + T, d), generator=gen, device=Hn.DEV) * (64 ** -0.25)).to(torch.bfloat16)
        v = torch.randn((P + T, d), generator=gen, device=Hn.DEV).to(torch.bfloat16)
        pg = pts[reqs[r][2]: reqs[r][2] + pages_per_req]
        vblocks = v.view(pages_per_req, pt, H, 64).permute(0, 2, 3, 1).contiguous()   # [page][head][d_h][token]
        kblocks = k.view(pages_per_req, pt, H, 64).permute(0, 2, 1, 3).contiguous()   # [page][head][token][d_h]
        base = torch.from_numpy(pg.astype(np.int64)).to(Hn.DEV) * (page // 2)
        for h in range(H):
            ko = Hn.kv_block_elem_offset(L, d, H, pt, 0, layer, 0, h)
            vo = Hn.kv_block_elem_offset(L, d, H, pt, 0, layer, 1, h)
            idx = base[:, None] + torch.arange(pt * 64, device=Hn.DEV)[None, :]
            mem[(idx + ko).reshape(-1)] = kblocks[:, h].reshape(-1)
            mem[(idx + vo).reshape(-1)] = vblocks[:, h].reshape(-1)
        if r in (0, 17):
            kv_host[r] = (k.float().cpu().numpy(), v.float().cpu().numpy())
    q = (torch.randn((N, d), generator=gen, device=Hn.DEV)).to(torch.bfloat16)
    o = torch.empty_like(q)
    rc = B.hstu_attn_paged(pool.h, model.h, layer, reqs, torch.from_numpy(pts).to(Hn.DEV), q,
                           torch.from_numpy(ts).to(Hn.DEV), o)
    assert rc == B.OK, B.last_error()
    torch.cuda.synchronize()
    assert pool.stats()["bad_pages"] == 0
    got = o.float().cpu().numpy()
    assert np.isfinite(got).all()
    # oracle on windows of query rows of two requests
    cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale, 1e-6, True)
    per_page = oracle.kv_elems_per_page(cfg)
    for r, (kk, vv) in kv_host.items():
        (P_, T_, pto, tso, xo) = reqs[r]
        okv = np.zeros(pages_per_req * per_page, dtype=np.float32)
        for j in range(P + T):  # the oracle's own layout, identity page table
            for h in range(H):
                ko = oracle.kv_offset(cfg, j // pt, layer, 0, h, j % pt)
                vo = oracle.kv_offset(cfg, j // pt, layer, 1, h, j % pt)
                okv[ko:ko + 64] = kk[j, h * 64:(h + 1) * 64]
                okv[vo:vo + 64] = vv[j, h * 64:(h + 1) * 64]
        qr = q[xo:xo + T].float().cpu().numpy().astype(np.float64)
        for i0 in (0, 250, 504):  # windows of 8 rows: first, middle, last
            ref = oracle.attn_paged(cfg, layer, w["pos"][layer], w["time"][layer], P + i0, 8,
                                    np.arange(pages_per_req, dtype=np.int32), ts[tso:tso + P + T], okv, qr[i0:i0 + 8])
            parity.assert_close(got[xo + i0: xo + i0 + 8], ref, True, "long history, attention alone, request %d rows %d.." % (r, i0))
    model.close()
    pool.close()


def test_long_history_config_whole_step_against_oracle():
    # Long history through hstu_step: 8 layers, d = 512, 8 heads, bf16; 32 requests x (16 384 cached + 512 new)
    # tokens, the cached K,V of every layer synthetic and written straight into shuffled pages.  The oracle
    # serves two of the requests (all 512 new tokens, all layers, all heads), one call each.
    L, d, H, pt, P, T, Bq = 8, 512, 8, 64, 16384, 512, 32
    n_pos, n_time, n_scale = 16896, 32, 16896.0
    rng = synth.rng_for(2, 1)
    w = synth.make_weights(rng, L, d, H, n_pos, n_time, True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, n_time, n_scale, w)
    page = model.page_size()
    pages_per_req = (P + T + pt - 1) // pt
    n_pages = ((Bq * pages_per_req * 4 // 3) // 32 + 1) * 32
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, None, 0.25)
    first_kv = n_pages // 4
    perm = first_kv + rng.permutation(n_pages - first_kv)
    reqs, n_pt, n_ts, N = synth.make_requests([P] * Bq, [T] * Bq, pt)
    pts = perm[:n_pt].astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng, P + T) for _ in range(Bq)])
    # the pool as [page][layer][K|V][head][pt * 64] (a K block is [token][d_h], a V block [d_h][token])
    mem = pool.mem.view(torch.bfloat16).view(n_pages, L, 2, H, pt * 64)
    gen = torch.Generator(device=Hn.DEV)
    gen.manual_seed(4321)
    sample = (3, 28)
    kv_host = {}
    for r in range(Bq):
        pg = torch.from_numpy(pts[reqs[r][2]: reqs[r][2] + pages_per_req].astype(np.int64)).to(Hn.DEV)
        for l in range(L):
            k = (torch.randn((P + T, d), generator=gen, device=Hn.DEV) * (64 ** -0.25)).to(torch.bfloat16)
            v = torch.randn((P + T, d), generator=gen, device=Hn.DEV).to(torch.bfloat16)
            mem[pg, l, 0] = k.view(pages_per_req, pt, H, 64).permute(0, 2, 1, 3).reshape(pages_per_req, H, pt * 64)
            mem[pg, l, 1] = v.view(pages_per_req, pt, H, 64).permute(0, 2, 3, 1).reshape(pages_per_req, H, pt * 64)
            if r in sample:
                kv_host[(r, l)] = (k.float().cpu().numpy(), v.float().cpu().numpy())
    x = synth.as_bf16_values(rng.standard_normal((N, d)).astype(np.float32))
    xd = torch.from_numpy(x).to(Hn.DEV).to(torch.bfloat16)
    out = torch.empty_like(xd)
    rc = B.hstu_step(pool.h, model.h, reqs, torch.from_numpy(pts).to(Hn.DEV), xd, torch.from_numpy(ts).to(Hn.DEV), out)
    assert rc == B.OK, B.last_error()
    torch.cuda.synchronize()
    assert pool.stats()["bad_pages"] == 0
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale, 1e-6, True)
    per_page = oracle.kv_elems_per_page(cfg)
    for r in sample:
        (P_, T_, pto, tso, xo) = reqs[r]
        # the oracle's own page layout ([layer][K|V][head][token][d_h]) under an identity page table
        okv = np.zeros((pages_per_req, L, 2, H, pt, 64), dtype=np.float32)
        for l in range(L):
            kk, vv = kv_host[(r, l)]
            okv[:, l, 0] = kk.reshape(pages_per_req, pt, H, 64).transpose(0, 2, 1, 3)
            okv[:, l, 1] = vv.reshape(pages_per_req, pt, H, 64).transpose(0, 2, 1, 3)
        okv = okv.reshape(-1)
        for (j, l, kvi, h) in ((0, 0, 0, 0), (16383, 7, 1, 5), (777, 3, 0, 7)):  # the layout above is the oracle's
            off = oracle.kv_offset(cfg, j // pt, l, kvi, h, j % pt)
            assert np.array_equal(okv[off:off + 64], kv_host[(r, l)][kvi][j, h * 64:(h + 1) * 64])
        rc, ref = oracle.hstu_step(cfg, w, [(P, T, 0, 0, 0)], np.arange(pages_per_req, dtype=np.int32), okv,
                                   x[xo:xo + T], ts[tso:tso + P + T])
        assert rc == oracle.OK
        parity.assert_close(got[xo:xo + T], ref, True, "long history, whole step, request %d" % r)
        # K,V of the new tokens as the last layer stored them
        pg = pts[pto:pto + pages_per_req]
        Kg, Vg = Hn.read_kv(pool.mem.view(torch.bfloat16), L, d, H, pt, pg, P + T, L - 1)
        o6 = okv.reshape(pages_per_req, L, 2, H, pt, 64)
        Ko = o6[:, L - 1, 0].transpose(0, 2, 1, 3).reshape(-1, d)[P:P + T]
        Vo = o6[:, L - 1, 1].transpose(0, 2, 1, 3).reshape(-1, d)[P:P + T]
        parity.assert_close(Kg[P:].float().cpu().numpy(), Ko, True, "long history, stored K of the new tokens")
        parity.assert_close(Vg[P:].float().cpu().numpy(), Vo, True, "long history, stored V of the new tokens")
    model.close()
    pool.close()


def test_mid_config_step_full_batch_short_and_longest_requests_against_oracle():
    # Mid model (4 layers, d = 256, 4 heads, bf16, 64-token pages) on the benchmark's batch of 64 lognormal
    # histories; the oracle recomputes the shortest requests in full (requests are independent)
    L, d, H, pt = 4, 256, 4, 64
    n_pos, n_time, n_scale = 8192, 32, 8192.0
    rng = synth.rng_for(1)
    lens = synth.history_lengths(rng, 64, 2048, 64, 8192)
    w = synth.make_weights(rng, L, d, H, n_pos, n_time, True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, n_time, n_scale, w)
    page = model.page_size()
    n_pages = 4096 + 1024
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, None, 0.2)
    reqs, n_pt, n_ts, N = synth.make_requests([0] * 64, lens, pt)
    pages = []
    for key, s in enumerate(lens):
        rc, pg = B.kv_seq_reserve(pool.h, key, int(s))
        assert rc == B.OK
        pages.append(pg)
    pts = np.concatenate(pages).astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng, int(s)) for s in lens])
    x = synth.as_bf16_values(rng.standard_normal((N, d)).astype(np.float32))
    xd = torch.from_numpy(x).to(Hn.DEV).to(torch.bfloat16)
    out = torch.empty_like(xd)
    rc = B.hstu_step(pool.h, model.h, reqs, torch.from_numpy(pts).to(Hn.DEV), xd, torch.from_numpy(ts).to(Hn.DEV), out)
    assert rc == B.OK, B.last_error()
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all() and pool.stats()["bad_pages"] == 0
    take = [int(r) for r in np.argsort(lens)[:6]]
    sub_lens = [int(lens[r]) for r in take]
    sreqs, s_pt, s_ts, sN = synth.make_requests([0] * len(take), sub_lens, pt)
    cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale, 1e-6, True)
    kv = np.zeros(s_pt * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    sx = np.concatenate([x[reqs[r][4]: reqs[r][4] + lens[r]] for r in take])
    sts = np.concatenate([ts[reqs[r][3]: reqs[r][3] + lens[r]] for r in take])
    rc, ref = oracle.hstu_step(cfg, w, sreqs, np.arange(s_pt, dtype=np.int32), kv, sx, sts)
    sg = np.concatenate([got[reqs[r][4]: reqs[r][4] + lens[r]] for r in take])
    parity.assert_close(sg, ref, True, "Mid, six shortest requests")
    # the longest request of the batch (several thousand tokens: its query tiles are cut into key ranges, it
    # is spread over the dies' work lists and sits in one of the three pipelines): the oracle serves it alone
    r = int(np.argmax(lens))
    S = int(lens[r])
    assert S >= 4096
    (P_, T_, pto, tso, xo) = reqs[r]
    lreqs, l_pt, l_ts, lN = synth.make_requests([0], [S], pt)
    kv = np.zeros(l_pt * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    rc, ref = oracle.hstu_step(cfg, w, lreqs, np.arange(l_pt, dtype=np.int32), kv, x[xo:xo + S], ts[tso:tso + S])
    parity.assert_close(got[xo:xo + S], ref, True, "Mid, longest request (%d tokens)" % S)
    # the same request served in two steps (prefix cached, then the tail) agrees with the one-step result
    cut = (S * 3 // 4) // 8 * 8 + 3
    ptd, tsd = torch.from_numpy(pts).to(Hn.DEV), torch.from_numpy(ts).to(Hn.DEV)
    o1 = torch.empty((cut, d), dtype=torch.bfloat16, device=Hn.DEV)
    o2 = torch.empty((S - cut, d), dtype=torch.bfloat16, device=Hn.DEV)
    assert B.hstu_step(pool.h, model.h, [(0, cut, pto, tso, 0)], ptd, xd[xo:xo + cut].contiguous(), tsd, o1) == B.OK
    assert B.hstu_step(pool.h, model.h, [(cut, S - cut, pto, tso, 0)], ptd, xd[xo + cut:xo + S].contiguous(), tsd, o2) == B.OK
    torch.cuda.synchronize()
    two = torch.cat([o1, o2]).float().cpu().numpy()
    err = parity.rel_error_rows(two, got[xo:xo + S])
    assert err.max() <= 2e-2, float(err.max())
    model.close()
    pool.close()


def test_split_sweep_config_pages_and_cache_follow_the_oracle():
    # Split sweep: 128 GiB pool of 256 KiB pages, table 100M x 256 bf16.  The hot cache is first filled at 0.8
    # with one refill sweep over the whole table (a dozen rows per set), then the EMB fraction walks the whole
    # grid 0.80, 0.75, .. 0.20 (every move evicts the least recently used entries of every set and compacts the
    # survivors out of the released pages: millions of rows move) and back up to 0.80, with a Zipf(0.9) lookup
    # batch after every move.  Hit flags, counters, tags, stamps and sampled resident rows follow the oracle;
    # resident KV sequences keep their pages and bytes.
    # (if the host cannot pin the 51.2 GB table, rows and pool are halved together, keeping the cache/table
    # ratio and the fraction grid; the scale actually used is printed)
    rows, d, pt, L = 100_000_000, 256, 64, 4
    pool_bytes = 128 << 30
    table = None
    for _ in range(4):
        table = pinned_bf16_table(rows, d, synth.SEED_BASE + 4, may_fail=True)
        if table is not None:
            break
        rows, pool_bytes = rows // 2, pool_bytes // 2
    if table is None:
        pytest.skip("cannot pin even a %d-row table" % (rows * 2))
    print("split sweep at %d table rows, %d GiB pool" % (rows, pool_bytes >> 30))
    page = pt * 2 * L * d * 2
    n_pages = pool_bytes // page
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), 0.8)
    orc = oracle.Pool(n_pages, pt, page // (d * 2), 32, 0.8)
    rng = synth.rng_for(4, 7)
    lens = synth.history_lengths(rng, 128, 4096, 512, 12288)
    kv_pages = {}
    marks = {}
    mem_pages = pool.mem.view(n_pages, page)
    for key, s in enumerate(lens[:24]):
        rc, pg = B.kv_seq_reserve(pool.h, key, int(s))
        assert rc == B.OK and np.array_equal(pg, orc.kv_reserve(key, int(s))[1])
        B.kv_seq_pin(pool.h, key)
        orc.kv_pin(key)
        kv_pages[key] = pg
        for k in (0, len(pg) - 1):
            mem_pages[int(pg[k])] = (key * 7 + k) % 251
            marks[(key, k)] = (key * 7 + k) % 251
    torch.cuda.synchronize()
    # fill: every row of the table once, in pieces (each piece is one refill batch, so stamps differ by piece)
    piece = 1 << 22
    for lo in range(0, rows, piece):
        n = min(piece, rows - lo)
        assert B.emb_refill(pool.h, torch.arange(lo, lo + n, dtype=torch.int64, device=Hn.DEV)) == B.OK, B.last_error()
        rc, ins = orc.emb_refill(np.arange(lo, lo + n, dtype=np.int64), rows)
        assert rc == oracle.OK
    filled = pool.stats()["inserted"]
    assert filled == orc.stats()["inserted"] and filled > 0.99 * rows
    n = 128 * 1024
    grid = [round(0.80 - 0.05 * k, 2) for k in range(13)]  # 0.80 .. 0.20
    walk = grid[1:] + grid[-2::-1]                        # down to 0.20, back up to 0.80
    for step, frac in enumerate(walk):
        rc, ach = B.pool_set_split(pool.h, frac)
        assert (rc, ach) == orc.set_split(frac), frac
        ids = synth.zipf_ids(rng, rows, 0.9, n)
        out, hit = pool.lookup(torch.from_numpy(ids).to(Hn.DEV))
        rc, _, ohit = orc.emb_lookup(ids, _rows_only(rows, d), want_out=False)
        assert np.array_equal(hit.cpu().numpy(), ohit), (frac, step)
        pick = rng.integers(0, n, size=2000)
        got = out[torch.from_numpy(pick).to(Hn.DEV)].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, table_rows_np(table, ids[pick])), (frac, step)
        st, so = pool.stats(), orc.stats()
        for k in ("hits", "misses", "inserted", "evicted", "bypassed", "shrink_evicted", "shrink_moved", "pages_emb"):
            assert st[k] == so[k], (frac, k, st[k], so[k])
        for (key, k), val in marks.items():  # KV pages never move and keep their bytes
            assert np.array_equal(B.kv_seq_lookup(pool.h, key)[2], kv_pages[key])
            assert bool((mem_pages[int(kv_pages[key][k])] == val).all()), (frac, key, k)
        if frac == grid[-1]:  # at the bottom of the walk: the whole cache state, rows included
            assert st["shrink_moved"] > rows // 100 and st["shrink_evicted"] > rows // 10, st
            check_cache_state(pool, orc, table)
    check_cache_state(pool, orc, table)
    pool.close()
