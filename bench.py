"""Benchmark of one HSTU serving step (emb_lookup + hstu_step) on one MI355X.

Default workload = the "Mid" configuration: 4 HSTU layers, d = 256, 4 heads, bf16; embedding
table 10M x 256 bf16 in pinned host memory; 64 GiB HBM pool of 256 KiB pages (64 KV tokens)
at EMB:KV = 0.5; batch of 64 requests with lognormal history lengths (mean 2048, max 8192);
Zipf(1.0) ids; every request is prefilled through its page table (prefix 0).

Prints ONE JSON line.  `--config tiny` runs the small fp32
configuration instead (used for quick checks).
"""
import argparse
import math
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0

CONFIGS = {
    # name: L, d, H, bf16, rows, pool_bytes, page_tokens, alpha, batch, mean_len, min_len, max_len, zipf_s, bag
    "mid": dict(index=1, L=4, d=256, H=4, bf16=True, rows=10_000_000, pool_bytes=64 << 30, pt=64, alpha=0.5,
                batch=64, mean_len=2048, min_len=64, max_len=8192, zipf=1.0, n_time=32, warm_batches=20,
                desc="Mid: 4 layers d=256 H=4 bf16, table 10Mx256 bf16 pinned host, 64 GiB pool @ EMB:KV=0.5, "
                     "batch 64 lognormal(mean 2048, max 8192) histories, Zipf(1.0), KV page 64 tokens"),
    # EMB-heavy: lookups only (8 sparse features per token, sum-pooled); shows the gather against HBM proper,
    # since a batch touches far more bytes than the caches hold
    "embheavy": dict(index=3, L=4, d=128, H=2, bf16=True, rows=100_000_000, pool_bytes=50 << 30, pt=64, alpha=0.8,
                     batch=256, mean_len=1024, min_len=1024, max_len=1024, zipf=0.8, n_time=32, warm_batches=3,
                     bag=8, emb_only=True,
                     desc="EMB-heavy: table 100Mx128 bf16 pinned host, 50 GiB pool @ EMB:KV=0.8 (40 GiB hot cache), "
                          "batch 256 x 1024 tokens x 8 features sum-pooled, Zipf(0.8); lookups only"),
    # A step that only appends: every request's history is cached, 64 new tokens each.  Every key tile is read once,
    # by one workgroup, so the attention kernel is measured against HBM here (K and V bytes of the histories)
    "append": dict(index=4, L=4, d=256, H=4, bf16=True, pt=64, batch=128, mean_len=3072, min_len=512, max_len=12288,
                   new=64, n_time=32, append_step=True,
                   desc="Append-only step: 4 layers d=256 H=4 bf16, 128 requests x 64 new tokens behind cached "
                        "lognormal(mean 3072, 512..12288) histories, KV page 64 tokens, pages shuffled"),
    # Several tables of different widths behind one hot cache: one lookup per table and token, all tables in one
    # launch (emb_lookup_tables) against one emb_lookup call per table; the cost per table is what the paper's
    # Sec. II-B observation (lookup time linear in the number of tables) is about
    "tables": dict(index=3, L=4, d=128, H=2, bf16=True, rows=2_000_000, pool_bytes=24 << 30, pt=64, alpha=0.8,
                   tokens=65536, zipf=0.8, n_tables=24, widths=(128, 64, 32), grid=(1, 2, 4, 8, 16, 24),
                   tables_bench=True,
                   desc="Tables: up to 24 tables of 2M rows x 128/64/32 bf16 (pinned host) behind one 19 GiB hot cache "
                        "of 256-byte slots, 65536 tokens x one Zipf(0.8) lookup per table; lookups only"),
    # Long history with KV reuse: the attention kernel alone (one layer) on 512 new tokens per request against a
    # 16k-token cached prefix held in shuffled pages
    "longreuse": dict(index=2, L=8, d=512, H=8, bf16=True, pt=64, batch=32, prefix=16384, new=512, n_time=32,
                      attn_only=True,
                      desc="Long history KV reuse: 8 layers d=512 H=8 bf16, 32 requests x (16384 cached + 512 new) tokens, "
                           "KV page 64 tokens; paged attention of one layer only"),
    # The same shape through hstu_step: all 8 layers, new K,V appended behind a cached prefix (random values stand in
    # for the cached keys and values; zeros would do for the arithmetic but let the chip clock higher)
    "longstep": dict(index=2, L=8, d=512, H=8, bf16=True, pt=64, batch=32, prefix=16384, new=512, n_time=32,
                     long_step=True,
                     desc="Long history KV reuse, whole step: 8 layers d=512 H=8 bf16, 32 requests x (16384 cached + 512 "
                          "new) tokens, KV page 64 tokens (1 MiB pages), pages shuffled"),
    # Split sweep: the boundary moves in steps of 0.05 down from 0.8 to 0.2 (each step evicts and compacts the
    # hot cache) and back up (metadata only), with lookup batches after every move
    "sweep": dict(index=4, L=4, d=256, H=4, bf16=True, rows=100_000_000, pool_bytes=128 << 30, pt=64, alpha=0.8,
                  batch=128, mean_len=3072, min_len=512, max_len=12288, zipf=0.9, n_time=32, split_sweep=True,
                  desc="Split sweep: 128 GiB pool, table 100Mx256 bf16 pinned host, EMB:KV 0.8 -> 0.2 -> 0.8 in steps of "
                       "0.05 with page remap/eviction, batches of 128 lognormal(512..12k) histories, Zipf(0.9) ids"),
    # Serving loop with KV reuse at every split of the grid: a request of a user whose history is still cached
    # computes its 64 newest tokens only, any other recomputes the whole history; lookups that miss the hot cache
    # go to the host table.  Half the size of the split-sweep configuration (pool, table and users scaled alike).
    "alphacurve": dict(index=5, L=4, d=256, H=4, bf16=True, rows=50_000_000, pool_bytes=64 << 30, pt=64, alpha=0.8,
                       batch=128, mean_len=3072, min_len=512, max_len=12288, zipf=0.9, n_time=32, alpha_curve=True,
                       users=8192, user_zipf=0.6, new=64, bag=8,
                       desc="Serving loop over the split grid 0.8 -> 0.2: 64 GiB pool, table 50Mx256 bf16 pinned host, "
                            "8192 users (Zipf 0.6 popularity, lognormal 512..12k histories), batches of 128 requests, "
                            "64 new tokens on a KV hit, full recompute otherwise, 8 sum-pooled features per token "
                            "(disjoint row ranges, Zipf(0.9) each)"),
    # Refill after growth: the hot cache grows from 0.2 to 0.5 of the pool (the new ways are empty) while lookup
    # batches keep coming; the empty ways are left to the live misses, filled at once, or filled a budget at a time
    "refill": dict(index=6, d=256, L=4, rows=50_000_000, pool_bytes=64 << 30, pt=64, alpha=0.8, zipf=0.9,
                   lookups=262144, batches=300, budget_mb=48, period_ms=4.0, refill_bench=True,
                   desc="Refill after growth 0.2 -> 0.5: 64 GiB pool, table 50Mx256 bf16 pinned host, batches of 262144 "
                        "Zipf(0.9) lookups arriving every 4 ms; no refill / one unthrottled refill / 48 MB of refill "
                        "per interval less the interval's live miss bytes"),
    # What the memory system grants: random row reads out of a 40 GiB region (no cache helps) and a plain copy.
    # The ceilings against which the gather and the other HBM-bound kernels are read.
    "hbmceiling": dict(index=7, region_bytes=40 << 30, read_bytes=2 << 30, hbm_ceiling=True,
                       desc="HBM ceilings: random reads of 128..1024-byte rows out of a 40 GiB region (read only, and "
                            "written out sequentially), and a sequential device copy of 2 GiB"),
    "tiny": dict(index=0, L=1, d=64, H=2, bf16=False, rows=100_000, pool_bytes=4 << 20, pt=16, alpha=0.5,
                 batch=4, mean_len=256, min_len=256, max_len=256, zipf=1.0, n_time=32, warm_batches=4,
                 desc="Tiny: 1 layer d=64 H=2 fp32, table 100k x 64 fp32, 4 MiB pool, 4 x 256 tokens, KV page 16"),
}


def measured_traffic(kernel, workload):
    """(HBM bytes per launch of `kernel`, where the figure comes from) out of the committed rocprofv3 counter summary,
    or (None, None).  The figure is not measured by this run: it is the summary's, and the source names the file and
    the commit the summary says it was taken at."""
    rel = os.path.join("profiles", "hbm_traffic_%s.txt" % workload)
    value, commit = None, "unknown commit"
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic.%s.%s=" % (kernel, workload)):
                value = float(line.split("=")[1])
            if line.startswith("measured_at_commit="):
                commit = line.split("=")[1].strip()
    except OSError:
        pass
    return (value, "%s @ %s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not re-measured by this run)" % (rel, commit)) \
        if value is not None else (None, None)


def build_workload(c, torch, Hn, B, synth):
    dev = Hn.DEV
    L, d, H, bf16, pt = c["L"], c["d"], c["H"], c["bf16"], c["pt"]
    esz = 2 if bf16 else 4
    elem = B.ELEM_BF16 if bf16 else B.ELEM_F32
    rng = synth.rng_for(c["index"])
    # host table (pinned)
    if bf16:
        table = torch.empty((c["rows"], d), dtype=torch.int16, pin_memory=True)
        synth.fill_table_bf16_torch(table, synth.SEED_BASE + c["index"], dev)
        table_t = table.view(torch.bfloat16)
    else:
        table_np = synth.make_table(rng, c["rows"], d, bf16=False)
        table_t = Hn.to_device_table(table_np)
    torch.cuda.synchronize()
    page_size = pt * 2 * L * d * esz
    n_pages = c["pool_bytes"] // page_size
    pool = Hn.Pool(n_pages, page_size, d * esz, elem, pt, 32, table_t, c["alpha"])
    lens = synth.history_lengths(rng, c["batch"], c["mean_len"], c["min_len"], c["max_len"])
    n_pos = c["max_len"]
    w = synth.make_weights(rng, L, d, H, n_pos, c["n_time"], bf16)
    model = Hn.Model(L, d, H, elem, pt, n_pos, c["n_time"], float(c["max_len"]), w)
    reqs, n_pt, n_ts, N = synth.make_requests([0] * len(lens), lens, pt)
    pages = []
    for key, s in enumerate(lens):
        rc, pg = B.kv_seq_reserve(pool.h, key, int(s))
        assert rc == B.OK, rc
        B.kv_seq_pin(pool.h, key)
        pages.append(pg)
    pts = np.concatenate(pages).astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng, int(s)) for s in lens])
    id_sets = [synth.zipf_ids(rng, c["rows"], c["zipf"], N) for _ in range(4)]
    wl = dict(pool=pool, model=model, table=table_t, lens=lens, reqs=reqs, N=N, weights=w,
              pts=pts, ts=ts, id_sets=id_sets, n_pos=n_pos, elem=elem, esz=esz, page_size=page_size, n_pages=n_pages)
    wl["pts_dev"] = torch.from_numpy(pts).to(dev)
    wl["ts_dev"] = torch.from_numpy(ts).to(dev)
    wl["ids_dev"] = [torch.from_numpy(a).to(dev) for a in id_sets]
    wl["reqs_c"] = (B.make_reqs(reqs), len(reqs))
    wl["x"] = torch.empty((N, d), dtype=Hn.torch_dtype(elem), device=dev)
    wl["out"] = torch.empty((N, d), dtype=Hn.torch_dtype(elem), device=dev)
    return wl


def emb_only_measure(args, c, torch, Hn, B, synth, steps=None):
    """Lookups only (pooled): whole emb_lookup calls per second and the probe+gather kernel against HBM.
    Returns the result line as a dict."""
    dev = Hn.DEV
    steps = steps or args.steps
    d, pt, L, bag = c["d"], c["pt"], c["L"], c["bag"]
    table = torch.empty((c["rows"], d), dtype=torch.int16, pin_memory=True)
    synth.fill_table_bf16_torch(table, synth.SEED_BASE + c["index"], dev)
    torch.cuda.synchronize()
    page_size = pt * 2 * L * d * 2
    n_pages = c["pool_bytes"] // page_size
    pool = Hn.Pool(n_pages, page_size, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), c["alpha"])
    rng = synth.rng_for(c["index"], 11)
    tokens = c["batch"] * c["mean_len"]
    n_sets = c["warm_batches"] + args.warmup + steps
    out = torch.empty((tokens, d), dtype=torch.bfloat16, device=dev)
    ids_dev = []
    for k in range(n_sets):
        ids_dev.append(torch.from_numpy(synth.multi_feature_ids(rng, c["rows"], bag, c["zipf"], tokens)).to(dev))
    # The hot cache of this configuration holds more slots than the table has rows, so its steady state is a
    # cache that has seen every row: reach it with one sweep over all ids (about the table's size over PCIe)
    # instead of thousands of Zipf batches, then settle with Zipf batches.
    per = tokens * bag
    for lo in range(0, c["rows"], per):
        sweep = torch.arange(lo, lo + per, dtype=torch.int64, device=dev) % c["rows"]
        rc = B.emb_lookup(pool.h, sweep, out, bag, None)
        assert rc == B.OK, (rc, B.last_error())
    for k in range(c["warm_batches"] + args.warmup):
        rc = B.emb_lookup(pool.h, ids_dev[k], out, bag, None)
        assert rc == B.OK, (rc, B.last_error())
    torch.cuda.synchronize()
    st0 = pool.stats()
    B.racer_prof_enable(pool.h, 1)
    B.racer_prof_read(pool.h)
    t0 = time.perf_counter()
    for k in range(steps):
        rc = B.emb_lookup(pool.h, ids_dev[c["warm_batches"] + args.warmup + k], out, bag, None)
        assert rc == B.OK, (rc, B.last_error())
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.racer_prof_read(pool.h)
    B.racer_prof_enable(pool.h, 0)
    st1 = pool.stats()
    lookups = st1["lookups"] - st0["lookups"]
    hits = st1["hits"] - st0["hits"]
    R = d * 2
    ways = st1["pages_emb"] / (n_pages / 32)
    # id + tag line + stamp per lookup, the row read of every hit, the pooled rows written
    gather_bytes = (lookups * (8 + 4 * ways + 4) + hits * R) / steps + tokens * R
    gather_ms = prof["emb_gather"][0] / max(prof["emb_gather"][1], 1)
    gbs = gather_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    # "useful" bytes: id, row read and the lookup's share of the pooled row written (no tag line, no stamp)
    useful_bytes = lookups * 8 / steps + hits * R / steps + tokens * R
    useful_gbs = useful_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    ms = dt * 1e3 / steps
    result = {
        "metric": "emb_lookup_tokens_per_s", "value": tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "tokens_per_step": tokens, "lookups_per_step": tokens * bag,
                   "hit_rate": hits / max(lookups, 1), "unique_misses_per_step": (st1["unique_misses"] - st0["unique_misses"]) / steps},
        "roofline": {"kernel": "emb_probe_gather", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": None, "bytes_per_launch": gather_bytes, "ms_per_launch": gather_ms,
                     "useful_GBps": useful_gbs, "useful_bytes_per_launch": useful_bytes},
        "kernels": {k: {"ms_per_launch": (v[0] / v[1] if v[1] else 0.0), "launches_per_step": v[1] / steps}
                    for k, v in prof.items() if v[1]},
    }
    pool.close()
    del pool, table, out, ids_dev
    return result


def emb_only_bench(args, c, torch, Hn, B, synth):
    print(json.dumps(emb_only_measure(args, c, torch, Hn, B, synth)))


def attn_only_bench(args, c, torch, Hn, B, synth):
    """The attention kernel of one layer on cached prefixes (synthetic K,V written straight into shuffled pages)."""
    dev = Hn.DEV
    L, d, H, pt, P, T, Bq = c["L"], c["d"], c["H"], c["pt"], c["prefix"], c["new"], c["batch"]
    n_pos = P + T
    rng = synth.rng_for(c["index"])
    w = synth.make_weights(rng, L, d, H, n_pos, c["n_time"], True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, c["n_time"], float(n_pos), w)
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
    mem = pool.mem.view(torch.bfloat16)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    for r in range(Bq):
        k = (torch.randn((P + T, d), generator=gen, device=dev) * (64 ** -0.25)).to(torch.bfloat16)
        v = torch.randn((P + T, d), generator=gen, device=dev).to(torch.bfloat16)
        pg = pts[reqs[r][2]: reqs[r][2] + pages_per_req]
        vblocks = v.view(pages_per_req, pt, H, 64).permute(0, 2, 3, 1).contiguous()   # [page][head][d_h][token]
        kblocks = k.view(pages_per_req, pt, H, 64).permute(0, 2, 1, 3).contiguous()   # [page][head][token][d_h]
        base = torch.from_numpy(pg.astype(np.int64)).to(dev) * (page // 2)
        idx = base[:, None] + torch.arange(pt * 64, device=dev)[None, :]
        for h in range(H):
            mem[(idx + Hn.kv_block_elem_offset(L, d, H, pt, 0, layer, 0, h)).reshape(-1)] = kblocks[:, h].reshape(-1)
            mem[(idx + Hn.kv_block_elem_offset(L, d, H, pt, 0, layer, 1, h)).reshape(-1)] = vblocks[:, h].reshape(-1)
    q = torch.randn((N, d), generator=gen, device=dev).to(torch.bfloat16)
    o = torch.empty_like(q)
    pts_dev, ts_dev = torch.from_numpy(pts).to(dev), torch.from_numpy(ts).to(dev)

    def call():
        rc = B.hstu_attn_paged(pool.h, model.h, layer, reqs, pts_dev, q, ts_dev, o)
        assert rc == B.OK, (rc, B.last_error())
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    B.racer_prof_enable(pool.h, 1)
    B.racer_prof_read(pool.h)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.racer_prof_read(pool.h)
    B.racer_prof_enable(pool.h, 0)
    pairs = float(Bq) * (T * P + T * (T + 1) / 2)
    flop = 4.0 * d * pairs
    attn_ms = prof["attention"][0] / max(prof["attention"][1], 1)
    tf = flop / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0
    ms = dt * 1e3 / args.steps
    print(json.dumps({
        "metric": "hstu_attention_tokens_per_s", "value": N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "new_tokens_per_step": int(N), "causal_pairs": pairs},
        "roofline": {"kernel": "attention_bf16_mfma", "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS, "traffic": None, "flop_per_launch": flop,
                     "ms_per_launch": attn_ms},
        "kernels": {k: {"ms_per_launch": (v[0] / v[1] if v[1] else 0.0), "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items() if v[1]},
    }))
    model.close()
    pool.close()


def long_step_bench(args, c, torch, Hn, B, synth):
    """hstu_step on cached prefixes: every layer's front half, paged attention against prefix + new keys, back half."""
    dev = Hn.DEV
    L, d, H, pt, P, T, Bq = c["L"], c["d"], c["H"], c["pt"], c["prefix"], c["new"], c["batch"]
    n_pos = P + T
    rng = synth.rng_for(c["index"])
    w = synth.make_weights(rng, L, d, H, n_pos, c["n_time"], True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, c["n_time"], float(n_pos), w)
    page = model.page_size()
    pages_per_req = (P + T + pt - 1) // pt
    n_pages = ((Bq * pages_per_req * 4 // 3) // 32 + 1) * 32
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, None, 0.25, zero_fill=False)
    first_kv = n_pages // 4
    perm = first_kv + rng.permutation(n_pages - first_kv)
    reqs, n_pt, n_ts, N = synth.make_requests([P] * Bq, [T] * Bq, pt)
    pts = torch.from_numpy(perm[:n_pt].astype(np.int32)).to(dev)
    ts = torch.from_numpy(np.concatenate([synth.timestamps(rng, P + T) for _ in range(Bq)])).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4321)
    for piece in pool.mem.view(torch.bfloat16).split(1 << 28):  # every page: N(0, 0.35^2) keys and values
        piece.copy_(torch.randn(piece.numel(), generator=gen, device=dev) * 0.35)
    x = (torch.randn((N, d), generator=gen, device=dev) * 0.5).to(torch.bfloat16)
    y = torch.empty_like(x)
    reqs_c = (B.make_reqs(reqs), len(reqs))

    def call():
        rc = B.hstu_step(pool.h, model.h, reqs_c, pts, x, ts, y)
        assert rc == B.OK, (rc, B.last_error())
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # once more with an event before and after every kernel, for the per-kernel durations
    B.racer_prof_enable(pool.h, 1)
    B.racer_prof_read(pool.h)
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    prof = B.racer_prof_read(pool.h)
    B.racer_prof_enable(pool.h, 0)
    pairs = float(Bq) * (T * P + T * (T + 1) / 2)
    flop = 4.0 * d * pairs
    attn_ms = prof["attention"][0] / max(prof["attention"][1], 1)
    tf = flop / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0
    ms = dt * 1e3 / args.steps
    print(json.dumps({
        "metric": "hstu_step_tokens_per_s", "value": N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "new_tokens_per_step": int(N), "causal_pairs_per_layer": pairs},
        "roofline": {"kernel": "attention_bf16_mfma", "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS, "traffic": None, "flop_per_launch": flop,
                     "ms_per_launch": attn_ms},
        "kernels": {k: {"ms_per_launch": (v[0] / v[1] if v[1] else 0.0), "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items() if v[1]},
    }))
    model.close()
    pool.close()


def split_sweep_bench(args, c, torch, Hn, B, synth):
    """pool_set_split over the alpha grid: time of each move (call + device work), rows evicted / moved, and the
    lookups that follow it (hit rate, time per batch including the miss path)."""
    dev = Hn.DEV
    d, pt, L = c["d"], c["pt"], c["L"]
    rows = c["rows"]
    import gc
    gc.collect()
    table = None
    while table is None:
        try:
            table = torch.empty((rows, d), dtype=torch.int16, pin_memory=True)
        except RuntimeError:
            rows //= 2  # the host cannot pin that much: halve the table (said in the output)
    synth.fill_table_bf16_torch(table, synth.SEED_BASE + c["index"], dev)
    torch.cuda.synchronize()
    page_size = pt * 2 * L * d * 2
    n_pages = c["pool_bytes"] // page_size
    pool = Hn.Pool(n_pages, page_size, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), c["alpha"], zero_fill=False)
    rng = synth.rng_for(c["index"], 5)
    lens = synth.history_lengths(rng, c["batch"], c["mean_len"], c["min_len"], c["max_len"])
    tokens = int(lens.sum())
    out = torch.empty((tokens, d), dtype=torch.bfloat16, device=dev)
    # warm: one sweep over the table (the cache at 0.8 holds more slots than the table has rows)
    for lo in range(0, rows, tokens):
        sweep = torch.arange(lo, lo + tokens, dtype=torch.int64, device=dev) % rows
        assert B.emb_lookup(pool.h, sweep, out, 1, None) == B.OK, B.last_error()
    torch.cuda.synchronize()
    R = d * 2
    grid = [round(0.8 - 0.05 * k, 2) for k in range(1, 13)] + [round(0.2 + 0.05 * k, 2) for k in range(1, 13)]
    steps = []
    for alpha in grid:
        st0 = pool.stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc, ach = B.pool_set_split(pool.h, alpha)
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        assert rc in (B.OK, B.DEFERRED), (rc, B.last_error())
        st1 = pool.stats()
        lk = []
        for k in range(args.steps):
            ids = torch.from_numpy(synth.zipf_ids(rng, rows, c["zipf"], tokens)).to(dev)
            torch.cuda.synchronize()
            ta = time.perf_counter()
            assert B.emb_lookup(pool.h, ids, out, 1, None) == B.OK, B.last_error()
            torch.cuda.synchronize()
            lk.append(time.perf_counter() - ta)
        st2 = pool.stats()
        lookups = st2["lookups"] - st1["lookups"]
        moved, evicted = st1["shrink_moved"] - st0["shrink_moved"], st1["shrink_evicted"] - st0["shrink_evicted"]
        steps.append({"alpha": alpha, "achieved": ach, "pages_moved": abs(int(st1["pages_emb"]) - int(st0["pages_emb"])),
                      "host_ms": (t1 - t0) * 1e3, "total_ms": (t2 - t0) * 1e3, "rows_evicted": int(evicted),
                      "rows_moved": int(moved), "moved_MB": 2 * R * moved / 1e6,
                      "hit_rate": (st2["hits"] - st1["hits"]) / max(lookups, 1),
                      "miss_MB_per_batch": (st2["unique_misses"] - st1["unique_misses"]) * R / 1e6 / args.steps,
                      "lookup_ms": 1e3 * sum(lk) / len(lk)})
    down = [s_ for s_ in steps[:12]]
    print(json.dumps({
        "metric": "pool_set_split_ms", "value": sum(s_["total_ms"] for s_ in down) / len(down), "unit": "ms per 0.05 shrink",
        "n_gpus": 1, "steps": args.steps, "warmup": 0, "ms_per_step": sum(s_["total_ms"] for s_ in down) / len(down),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": c["desc"], "table_rows": rows, "pages": int(n_pages), "lookups_per_batch": tokens},
        "moves": steps}))
    pool.close()


def alpha_curve_bench(args, c, torch, Hn, B, synth):
    """Step time of a serving loop against the EMB:KV split (the trade-off of the paper's Sec. III, Fig. 4): the
    embedding side gets slower as the hot cache shrinks (misses cross PCIe), the attention side gets slower as
    the KV share shrinks (fewer users stay cached, their histories are recomputed).  One curve per mean history
    length; per split: KV hit rate, cache hit rate, miss bytes, time of emb_lookup and of hstu_step."""
    dev = Hn.DEV
    L, d, H, pt = c["L"], c["d"], c["H"], c["pt"]
    rows = c["rows"]
    table = None
    while table is None:
        try:
            table = torch.empty((rows, d), dtype=torch.int16, pin_memory=True)
        except RuntimeError:
            rows //= 2  # the host cannot pin that much: halve the table (said in the output)
    synth.fill_table_bf16_torch(table, synth.SEED_BASE + c["index"], dev)
    torch.cuda.synchronize()
    page_size = pt * 2 * L * d * 2
    n_pages = c["pool_bytes"] // page_size
    n_pos = c["max_len"]
    rng = synth.rng_for(c["index"])
    w = synth.make_weights(rng, L, d, H, n_pos, c["n_time"], True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, c["n_time"], float(n_pos), w)
    ts_all = synth.timestamps(rng, c["max_len"])
    users, new = c["users"], c["new"]
    pop = np.arange(1, users + 1, dtype=np.float64) ** (-c["user_zipf"])
    pop /= pop.sum()
    grid = [round(0.8 - 0.05 * k, 2) for k in range(13)]
    curves = []
    for mean_len in (c["mean_len"] * 2 // 3, c["mean_len"] * 4 // 3):
        pool = Hn.Pool(n_pages, page_size, d * 2, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), c["alpha"],
                       zero_fill=True)
        lens = synth.history_lengths(rng, users, mean_len, c["min_len"], c["max_len"])
        user_of_rank = rng.permutation(users)
        sweep_n = 1 << 19
        out_sweep = torch.empty((sweep_n, d), dtype=torch.bfloat16, device=dev)
        per = rows // c["bag"]  # the hottest rows of every feature range, hottest first, for refills after a growth
        hot = torch.from_numpy((synth.ranks_to_rows(np.arange(1, per + 1), per)[:, None]
                                + np.arange(c["bag"], dtype=np.int64)[None, :] * per).reshape(-1)).to(dev)
        # warm the hot cache: one pass over the table, then a Zipf stream that sets the LRU order
        for lo in range(0, rows, sweep_n):
            ids = torch.arange(lo, lo + sweep_n, dtype=torch.int64, device=dev) % rows
            assert B.emb_lookup(pool.h, ids, out_sweep, 1, None) == B.OK, B.last_error()
        for _ in range(40):
            ids = torch.from_numpy(synth.multi_feature_ids(rng, rows, c["bag"], c["zipf"], sweep_n // c["bag"])).to(dev)
            assert B.emb_lookup(pool.h, ids, out_sweep, 1, None) == B.OK, B.last_error()
        torch.cuda.synchronize()

        def serve(timed):
            """One batch; returns (requests, KV hits, new tokens, emb s, hstu s)."""
            picked = np.unique(user_of_rank[rng.choice(users, size=c["batch"], p=pop)])
            prefix, newt, pages, keys = [], [], [], []
            for u in picked:
                S = int(lens[u])
                rc, tok, _ = B.kv_seq_lookup(pool.h, int(u))
                hit = rc == B.OK and tok >= S
                rc, pg = B.kv_seq_reserve(pool.h, int(u), S)
                if rc != B.OK:
                    continue  # the KV side cannot hold this batch: the request is dropped (counted below)
                B.kv_seq_pin(pool.h, int(u))
                keys.append(int(u))
                prefix.append(S - new if hit else 0)
                newt.append(new if hit else S)
                pages.append(pg[: (S + pt - 1) // pt])
            reqs, n_pt, n_ts, N = synth.make_requests(prefix, newt, pt)
            pts = torch.from_numpy(np.concatenate(pages).astype(np.int32)).to(dev)
            ts = torch.from_numpy(np.concatenate([ts_all[: p_ + t_] for p_, t_ in zip(prefix, newt)])).to(dev)
            ids = torch.from_numpy(synth.multi_feature_ids(rng, rows, c["bag"], c["zipf"], N)).to(dev)
            x = torch.empty((N, d), dtype=torch.bfloat16, device=dev)
            y = torch.empty((N, d), dtype=torch.bfloat16, device=dev)
            reqs_c = (B.make_reqs(reqs), len(reqs))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rc = B.emb_lookup(pool.h, ids, x, c["bag"], None)
            assert rc == B.OK, (rc, B.last_error())
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            rc = B.hstu_step(pool.h, model.h, reqs_c, pts, x, ts, y)
            assert rc == B.OK, (rc, B.last_error())
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for k_ in keys:
                B.kv_seq_unpin(pool.h, k_)
            hits = sum(1 for p_ in prefix if p_ > 0)
            return len(picked), len(keys), hits, N, t1 - t0, t2 - t1

        def measure(alpha, tag):
            """Move the boundary (refilling what a growth left empty), let the caches settle, time args.steps batches."""
            grows = alpha > pool.stats()["pages_emb"] / n_pages + 1e-6
            rc, ach = B.pool_set_split(pool.h, alpha)
            assert rc in (B.OK, B.DEFERRED), (rc, B.last_error())
            if grows:
                slots = int(pool.stats()["pages_emb"]) * (page_size // (d * 2))
                for lo in range(0, min(slots, hot.numel()), sweep_n):
                    assert B.emb_refill(pool.h, hot[lo: lo + sweep_n]) == B.OK, B.last_error()
            for _ in range(args.warmup):
                serve(False)
            st0 = pool.stats()
            acc = np.zeros(6)
            for _ in range(args.steps):
                acc += np.array(serve(True), dtype=np.float64)
            st1 = pool.stats()
            lookups = st1["lookups"] - st0["lookups"]
            pt_ = {"alpha": alpha, "achieved": ach, "kv_hit_rate": acc[2] / max(acc[1], 1),
                   "dropped_requests": int(acc[0] - acc[1]),
                   "emb_hit_rate": (st1["hits"] - st0["hits"]) / max(lookups, 1),
                   "miss_MB_per_step": (st1["unique_misses"] - st0["unique_misses"]) * d * 2 / 1e6 / args.steps,
                   "new_tokens_per_step": acc[3] / args.steps, "emb_ms": 1e3 * acc[4] / args.steps,
                   "hstu_ms": 1e3 * acc[5] / args.steps, "total_ms": 1e3 * (acc[4] + acc[5]) / args.steps}
            print("alphacurve mean %d %s: %s" % (mean_len, tag, json.dumps(pt_)), file=sys.stderr, flush=True)
            return pt_

        points = [measure(alpha, "grid") for alpha in grid]
        best = min(points, key=lambda q: q["total_ms"])
        # Closed loop: the library's split controller (paper Sec. IV-A: action set {+-0.06, +-0.04, +-0.02, 0} of
        # Eq. 3, alpha <- clip(alpha + step, 0.1, 0.9) of Eq. 6; its policy is a hill climb on the measured latency,
        # a stand-in for the paper's trained policy), one decision per measured window, started at 0.8
        ctl = B.AlphaController(slo_ms=30.0)
        alpha, path = 0.8, []
        for epoch in range(24):
            cur = measure(alpha, "ctl")
            step, nxt, burst = ctl.decide(alpha, float(cur["total_ms"]), kv_hit_rate=float(cur["kv_hit_rate"]),
                                          emb_hit_rate=float(cur["emb_hit_rate"]), mean_seq_len=float(mean_len))
            path.append({"alpha": alpha, "total_ms": float(cur["total_ms"]), "step": step, "burst": burst})
            alpha = round(nxt, 2)
        ctl.close()
        curves.append({"mean_history": int(mean_len), "best_alpha": best["alpha"], "best_total_ms": best["total_ms"],
                       "points": points, "controller_path": path, "controller_alpha": alpha})
        pool.close()
        del pool, out_sweep, hot
    print(json.dumps({
        "metric": "serving_step_ms_at_best_split", "value": curves[0]["best_total_ms"], "unit": "ms per batch of %d requests" % c["batch"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": curves[0]["best_total_ms"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "table_rows": rows, "pages": int(n_pages)}, "curves": curves}))
    model.close()


def refill_bench(args, c, torch, Hn, B, synth):
    """Latency of live lookup batches while the empty ways of a grown hot cache are refilled (paper Sec. IV-B: the
    refill shares the host link with the live misses and is throttled against them).  Batches arrive at a fixed
    period; refill work is queued behind a batch for the gap before the next one.  Three policies from the same
    starting state; per policy the batch latency (arrival to completion), the hit rate over time and the bytes each
    side moved."""
    dev = Hn.DEV
    d, pt, L = c["d"], c["pt"], c["L"]
    rows = c["rows"]
    table = None
    while table is None:
        try:
            table = torch.empty((rows, d), dtype=torch.int16, pin_memory=True)
        except RuntimeError:
            rows //= 2  # the host cannot pin that much: halve the table (said in the output)
    synth.fill_table_bf16_torch(table, synth.SEED_BASE + c["index"], dev)
    torch.cuda.synchronize()
    R = d * 2
    page_size = pt * 2 * L * d * 2
    n_pages = c["pool_bytes"] // page_size
    n, K = c["lookups"], c["batches"]
    out = torch.empty((n, d), dtype=torch.bfloat16, device=dev)
    hot = torch.from_numpy(synth.ranks_to_rows(np.arange(1, rows + 1), rows)).to(dev)  # every row, hottest first
    chunk = 65536  # ids per refill call: at most 32 MB over the link
    results = []
    for policy in ("none", "unthrottled", "throttled"):
        rng = synth.rng_for(c["index"], 1)  # the same id stream for every policy
        pool = Hn.Pool(n_pages, page_size, R, B.ELEM_BF16, pt, 32, table.view(torch.bfloat16), c["alpha"], zero_fill=False)
        for lo in range(0, rows, n):  # every row once, then a Zipf stream that sets the LRU order
            assert B.emb_lookup(pool.h, hot[lo: lo + n], out, 1, None) == B.OK, B.last_error()
        warm = [torch.from_numpy(synth.zipf_ids(rng, rows, c["zipf"], n)).to(dev) for _ in range(30)]
        for ids in warm:
            assert B.emb_lookup(pool.h, ids, out, 1, None) == B.OK, B.last_error()
        assert B.pool_set_split(pool.h, 0.2)[0] == B.OK
        for ids in warm[:10]:
            assert B.emb_lookup(pool.h, ids, out, 1, None) == B.OK, B.last_error()
        rc, ach = B.pool_set_split(pool.h, 0.5)
        assert rc == B.OK, (rc, B.last_error())
        torch.cuda.synchronize()
        batches = [torch.from_numpy(synth.zipf_ids(rng, rows, c["zipf"], n)).to(dev) for _ in range(K)]
        st0 = pool.stats()
        cursor, budget_rows = 0, c["budget_mb"] * 1000000 // R
        lat, hit_rate = [], []
        prev, live_last, yield_last, refill_rows = st0, 0, 1.0, 0
        t_begin = time.perf_counter()
        period = c["period_ms"] * 1e-3
        issued = 0
        for k in range(K):
            # batch k arrives at t_begin + k * period whatever the device is doing; its latency runs from then
            arrival = t_begin + k * period
            while time.perf_counter() < arrival:
                pass
            assert B.emb_lookup(pool.h, batches[k], out, 1, None) == B.OK, B.last_error()
            torch.cuda.synchronize()
            lat.append(time.perf_counter() - arrival)
            st = pool.stats()
            hit_rate.append((st["hits"] - prev["hits"]) / n)
            live_last = st["unique_misses"] - prev["unique_misses"]
            entered = (st["inserted"] - prev["inserted"]) - (live_last - (st["bypassed"] - prev["bypassed"]))
            refill_rows += entered
            if issued:
                yield_last = entered / issued
            prev = st
            # refill work for the gap before the next arrival (it runs behind this batch on the same stream)
            if policy == "unthrottled" and k == 0:
                want = rows
            elif policy == "throttled":
                # the interval's budget, less what the live misses of this batch took from the link, in ids:
                # the last interval's yield (rows that entered per id offered) turns rows into ids
                want = int(max(budget_rows - live_last, 0) / max(yield_last, 0.05))
            else:
                want = 0
            issued = 0
            while cursor < rows and issued < want:
                assert B.emb_refill(pool.h, hot[cursor: cursor + chunk]) == B.OK, B.last_error()
                issued += min(chunk, rows - cursor)
                cursor += chunk
        total_s = time.perf_counter() - t_begin
        st1 = pool.stats()
        live_rows = st1["unique_misses"] - st0["unique_misses"]
        refilled = refill_rows
        lat_ms = np.array(lat) * 1e3
        reach = next((k for k, h in enumerate(hit_rate) if h >= 0.999), None)
        results.append({"policy": policy, "p50_ms": float(np.percentile(lat_ms, 50)), "p99_ms": float(np.percentile(lat_ms, 99)),
                        "max_ms": float(lat_ms.max()), "total_s": total_s, "first_hit_rate": hit_rate[0],
                        "last_hit_rate": hit_rate[-1], "batches_to_0.999": reach,
                        "live_miss_MB": live_rows * R / 1e6, "refill_MB": refilled * R / 1e6})
        print("refill %s" % json.dumps(results[-1]), file=sys.stderr, flush=True)
        pool.close()
        del pool
    thr = results[2]
    print(json.dumps({
        "metric": "emb_lookup_p99_ms_during_throttled_refill", "value": thr["p99_ms"], "unit": "ms per batch of %d lookups" % n,
        "n_gpus": 1, "steps": K, "warmup": 0, "ms_per_step": thr["p50_ms"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": c["desc"], "table_rows": rows, "pages": int(n_pages), "budget_MB_per_interval": c["budget_mb"]},
        "policies": results}))


def hbm_ceiling_bench(args, c, torch, Hn, B, synth):
    """Rates of racer_hbm_probe (random row reads) and of a plain device copy, HIP events around each launch."""
    dev = Hn.DEV
    region = torch.empty(c["region_bytes"], dtype=torch.uint8, device=dev)
    for piece in region.split(1 << 30):
        piece.fill_(1)
    out = torch.empty(c["read_bytes"], dtype=torch.uint8, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def timed(fn):
        for _ in range(max(args.warmup, 1)):
            fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(max(args.steps, 1)):
            ev[0].record()
            fn()
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1])
            best = ms if best is None else min(best, ms)
        return best

    rows = []
    seed = [1]
    for row_bytes in (128, 256, 512, 1024):
        n_reads = c["read_bytes"] // row_bytes
        for write in (False, True):
            def fn():
                seed[0] += 1
                rc = B.racer_hbm_probe(region, row_bytes, n_reads, out if write else None, seed[0])
                assert rc == B.OK, rc
            ms = timed(fn)
            moved = c["read_bytes"] * (2 if write else 1)
            rows.append({"row_bytes": row_bytes, "written_out": write, "ms": ms, "GBps": moved / ms / 1e6,
                         "frac_of_hbm_peak": moved / ms / 1e6 / PEAK_HBM_GBS})
            print("random rows of %4d B, %s: %.3f ms, %.0f GB/s" % (row_bytes, "read + write" if write else "read only", ms,
                                                                     moved / ms / 1e6), file=sys.stderr, flush=True)
    src = region[: c["read_bytes"]]
    ms = timed(lambda: out.copy_(src))
    copy_gbs = 2 * c["read_bytes"] / ms / 1e6
    best_read = max(r["GBps"] for r in rows if not r["written_out"])
    print(json.dumps({
        "metric": "hbm_random_row_read_GBps", "value": best_read, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": min(r["ms"] for r in rows if not r["written_out"]), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": c["desc"]},
        "roofline": {"kernel": "random_row_reads", "bound": "hbm", "achieved": best_read, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": best_read / PEAK_HBM_GBS, "traffic": None},
        "random_rows": rows,
        "sequential_copy": {"bytes_read_plus_written": 2 * c["read_bytes"], "ms": ms, "GBps": copy_gbs,
                            "frac_of_hbm_peak": copy_gbs / PEAK_HBM_GBS}}))


def one_step(wl, k, B):
    ids = wl["ids_dev"][k % len(wl["ids_dev"])]
    rc = B.emb_lookup(wl["pool"].h, ids, wl["x"], 1, None)
    assert rc == B.OK, (rc, B.last_error())
    rc = B.hstu_step(wl["pool"].h, wl["model"].h, wl["reqs_c"], wl["pts_dev"], wl["x"], wl["ts_dev"], wl["out"])
    assert rc == B.OK, (rc, B.last_error())


def cpu_baseline(c, wl, synth, budget_tokens):
    """Time the oracle on a bounded sample: requests taken in batch order (so short and long histories come as the
    batch has them) until their causal (query, key) pairs reach the batch's pairs-per-token ratio times
    `budget_tokens`, served as their own small step (EMB lookup + all layers)."""
    import oracle
    L, d, H, pt, bf16 = c["L"], c["d"], c["H"], c["pt"], c["bf16"]
    lens = [int(s) for s in wl["lens"]]
    pairs_of = lambda s: s * (s + 1) // 2
    budget_pairs = budget_tokens * sum(pairs_of(s) for s in lens) / max(sum(lens), 1)
    take, tot = [], 0
    for r in range(len(lens)):
        if tot + pairs_of(lens[r]) > budget_pairs and take:
            continue  # too long for what is left of the budget: try the next one
        take.append(r)
        tot += pairs_of(lens[r])
    sub_lens = [lens[r] for r in take]
    reqs, n_pt, n_ts, N = synth.make_requests([0] * len(take), sub_lens, pt)
    pts = np.arange(n_pt, dtype=np.int32)
    ts = np.concatenate([wl["ts"][wl["reqs"][r][3]: wl["reqs"][r][3] + lens[r]] for r in take])
    ids = np.concatenate([wl["id_sets"][0][wl["reqs"][r][4]: wl["reqs"][r][4] + lens[r]] for r in take])
    # the oracle's table: only the sampled rows are materialised (row -> dense index), same values
    uniq, inv = np.unique(ids, return_inverse=True)
    if bf16:
        sub = np.zeros((len(uniq), d), dtype=np.uint16)
        tab = wl["table"].view(dtype=__import__("torch").int16)
        sub[:] = tab[__import__("torch").from_numpy(uniq)].numpy().view(np.uint16)
        x_vals = synth.from_bf16_bits(sub)
    else:
        sub = wl["table"][__import__("torch").from_numpy(uniq)].numpy()
        x_vals = sub
    orc_pool = oracle.Pool((2 * len(uniq) // 1024 + 2) * 32, pt, 32, 32, 0.5)  # capacity >= the distinct rows
    cfg = oracle.make_cfg(L, d, H, pt, wl["n_pos"], c["n_time"], float(c["max_len"]), 1e-6, bf16)
    kv = np.zeros(n_pt * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    rc, xo, hit = orc_pool.emb_lookup(inv.astype(np.int64), sub)
    x = synth.from_bf16_bits(xo) if bf16 else xo
    rc, ref = oracle.hstu_step(cfg, wl["weights"], reqs, pts, kv, x, ts, threads=0)
    dt = time.perf_counter() - t0
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    cb = {"value": N / dt, "unit": "tokens/s", "cores": min(threads, len(take)), "kind": "oracle",
          "wall_s": dt, "cpu_model": cpu_model,
          "sample": "%d requests of the batch in batch order (%d tokens, %.0f causal pairs per token against %.0f for the "
                    "whole batch), EMB lookup + all %d layers, %.1f s, OpenMP over requests (%d threads available)"
                    % (len(take), N, tot / max(N, 1), sum(pairs_of(s) for s in lens) / max(sum(lens), 1), L, dt, threads)}
    return cb, take, ref


def append_step_bench(args, c, torch, Hn, B, synth):
    """hstu_step on a batch whose histories are all cached: 64 new tokens per request."""
    dev = Hn.DEV
    L, d, H, pt, Bq, T = c["L"], c["d"], c["H"], c["pt"], c["batch"], c["new"]
    rng = synth.rng_for(c["index"] + 1)
    lens = synth.history_lengths(rng, Bq, c["mean_len"], c["min_len"], c["max_len"])
    n_pos = c["max_len"]
    w = synth.make_weights(rng, L, d, H, n_pos, c["n_time"], True)
    model = Hn.Model(L, d, H, B.ELEM_BF16, pt, n_pos, c["n_time"], float(n_pos), w)
    page = model.page_size()
    need = int(sum((int(s_) + pt - 1) // pt for s_ in lens))
    n_pages = ((need * 4 // 3) // 32 + 1) * 32
    pool = Hn.Pool(n_pages, page, d * 2, B.ELEM_BF16, pt, 32, None, 0.25, zero_fill=True)
    first_kv = n_pages // 4
    perm = first_kv + rng.permutation(n_pages - first_kv)
    prefix = [int(s_) - T for s_ in lens]
    reqs, n_pt, n_ts, N = synth.make_requests(prefix, [T] * Bq, pt)
    pts = torch.from_numpy(perm[:n_pt].astype(np.int32)).to(dev)
    ts_all = synth.timestamps(rng, c["max_len"])
    ts = torch.from_numpy(np.concatenate([ts_all[:int(s_)] for s_ in lens])).to(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4322)
    for piece in pool.mem.view(torch.bfloat16).split(1 << 28):  # every page: N(0, 0.35^2) keys and values
        piece.copy_(torch.randn(piece.numel(), generator=gen, device=dev) * 0.35)
    x = (torch.randn((N, d), generator=gen, device=dev) * 0.5).to(torch.bfloat16)
    y = torch.empty_like(x)
    reqs_c = (B.make_reqs(reqs), len(reqs))

    def call():
        rc = B.hstu_step(pool.h, model.h, reqs_c, pts, x, ts, y)
        assert rc == B.OK, (rc, B.last_error())
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.racer_prof_enable(pool.h, 1)
    B.racer_prof_read(pool.h)
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    prof = B.racer_prof_read(pool.h)
    B.racer_prof_enable(pool.h, 0)
    pairs = float(sum(T * p_ + T * (T + 1) / 2 for p_ in prefix))
    attn_ms = prof["attention"][0] / max(prof["attention"][1], 1)
    # K and V of every key of every request, all heads of one layer: 2 * d elements per key
    kv_bytes = float(sum(int(s_) for s_ in lens)) * 2 * d * 2
    gbs = kv_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms > 0 else 0.0
    ms = dt * 1e3 / args.steps
    print(json.dumps({
        "metric": "hstu_step_tokens_per_s", "value": N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "new_tokens_per_step": int(N), "mean_history": float(np.mean(lens)),
                   "causal_pairs_per_layer": pairs},
        "roofline": {"kernel": "attention_bf16_mfma", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": None, "bytes_per_launch": kv_bytes,
                     "ms_per_launch": attn_ms, "mfma_tflops": 4.0 * d * pairs / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0},
        "kernels": {k: {"ms_per_launch": (v[0] / v[1] if v[1] else 0.0), "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items() if v[1]},
    }))
    model.close()
    pool.close()


def tables_bench(args, c, torch, Hn, B, synth):
    """emb_lookup_tables over a growing number of tables: one launch for all against one emb_lookup per table."""
    dev = Hn.DEV
    d, pt, L, rows, tokens = c["d"], c["pt"], c["L"], c["rows"], c["tokens"]
    T_max = c["n_tables"]
    widths = [c["widths"][t % len(c["widths"])] for t in range(T_max)]
    tables = []
    for t in range(T_max):
        tab = torch.empty((rows, widths[t]), dtype=torch.int16, pin_memory=True)
        synth.fill_table_bf16_torch(tab, synth.SEED_BASE + 100 * c["index"] + t, dev)
        tables.append(tab)
    torch.cuda.synchronize()
    page_size = pt * 2 * L * d * 2
    n_pages = c["pool_bytes"] // page_size
    pool = Hn.Pool(n_pages, page_size, d * 2, B.ELEM_BF16, pt, 32, tables[0].view(torch.bfloat16), c["alpha"])
    for t in range(1, T_max):
        rc, num = B.pool_add_table(pool.h, tables[t].view(torch.bfloat16), rows, widths[t] * 2)
        assert (rc, num) == (B.OK, t), (rc, B.last_error())
    # steady state = a cache that has seen every row (it has more slots than the tables have rows)
    per = 1 << 21
    sweep_out = torch.empty((per, d), dtype=torch.bfloat16, device=dev)
    for lo in range(0, T_max * rows, per):
        n = min(per, T_max * rows - lo)
        rc = B.emb_lookup(pool.h, torch.arange(lo, lo + n, dtype=torch.int64, device=dev), sweep_out[:n], 1, None)
        assert rc == B.OK, (rc, B.last_error())
    torch.cuda.synchronize()
    del sweep_out
    rng = synth.rng_for(c["index"], 17)
    n_sets = 4
    out = torch.empty((tokens * T_max, d), dtype=torch.bfloat16, device=dev)
    per_tables = []
    for T in c["grid"]:
        # ids[k]: [token][table] rows inside their tables; the same lookups table after table for the separate calls
        ids_tok, ids_tab = [], []
        for k in range(n_sets):
            cols = np.stack([synth.zipf_ids(rng, rows, c["zipf"], tokens) for _ in range(T)], axis=1)
            ids_tok.append(torch.from_numpy(cols.reshape(-1).astype(np.int64)).to(dev))
            glob = cols + np.arange(T, dtype=np.int64)[None, :] * rows
            ids_tab.append(torch.from_numpy(np.ascontiguousarray(glob.T).astype(np.int64)).to(dev))
        table_of = torch.arange(T, dtype=torch.int32, device=dev).repeat(tokens)
        n = tokens * T

        def one_launch(k):
            rc = B.emb_lookup_tables(pool.h, table_of, ids_tok[k % n_sets], out[:n], 1, None)
            assert rc == B.OK, (rc, B.last_error())

        def per_table(k):
            for t in range(T):
                rc = B.emb_lookup(pool.h, ids_tab[k % n_sets][t], out[t * tokens:(t + 1) * tokens], 1, None)
                assert rc == B.OK, (rc, B.last_error())

        res = {}
        for name, fn in (("one_launch", one_launch), ("per_table", per_table)):
            for k in range(args.warmup):
                fn(k)
            torch.cuda.synchronize()
            st0 = pool.stats()
            t0 = time.perf_counter()
            for k in range(args.steps):
                fn(k)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            st1 = pool.stats()
            res[name] = {"ms_per_step": ms, "us_per_table": ms * 1e3 / T,
                         "hit_rate": (st1["hits"] - st0["hits"]) / max(st1["lookups"] - st0["lookups"], 1)}
        per_tables.append({"tables": T, "lookups_per_step": n, **res})
        print("tables %2d: one launch %.3f ms, one call per table %.3f ms" %
              (T, res["one_launch"]["ms_per_step"], res["per_table"]["ms_per_step"]), file=sys.stderr, flush=True)
    last = per_tables[-1]
    ms = last["one_launch"]["ms_per_step"]
    result = {
        "metric": "emb_lookup_tables_lookups_per_s", "value": last["lookups_per_step"] / (ms * 1e-3), "unit": "lookups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["desc"], "tokens_per_step": tokens, "tables": last["tables"]},
        "per_tables": per_tables,
    }
    print(json.dumps(result))
    pool.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="mid", choices=sorted(CONFIGS))
    ap.add_argument("--cpu-tokens", type=int, default=None, help="token budget of the oracle sample")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-embheavy", action="store_true",
                    help="leave out the EMB-heavy lookups-only pass (the gather against HBM proper) that the default run appends")
    ap.add_argument("--one-pipeline", action="store_true",
                    help="run the throughput pass as one pipeline as well (per-kernel events on): every kernel launch "
                         "then covers the whole batch, which is what a per-kernel profile of the run needs")
    ap.add_argument("--copy-calib-mb", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "traffic against which HBM byte counters of a profiler run are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (every figure is the one "
              "GPU's throughput)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_04450_amd import binding as B
    from paper_2605_04450_amd import device as Hn
    from paper_2605_04450_amd import synth

    B.load()
    c = CONFIGS[args.config]
    if c.get("emb_only"):
        emb_only_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("attn_only"):
        attn_only_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("long_step"):
        long_step_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("split_sweep"):
        split_sweep_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("alpha_curve"):
        alpha_curve_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("refill_bench"):
        refill_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("tables_bench"):
        tables_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("append_step"):
        append_step_bench(args, c, torch, Hn, B, synth)
        return
    if c.get("hbm_ceiling"):
        hbm_ceiling_bench(args, c, torch, Hn, B, synth)
        return
    wl = build_workload(c, torch, Hn, B, synth)
    pool = wl["pool"]
    # warm the EMB cache, then whole warm-up steps
    for k in range(c["warm_batches"]):
        B.emb_lookup(pool.h, wl["ids_dev"][k % 4], wl["x"], 1, None)
    if args.one_pipeline:
        B.racer_prof_enable(pool.h, 1)
    for k in range(args.warmup):
        one_step(wl, k, B)
    torch.cuda.synchronize()
    B.racer_prof_read(pool.h)
    st0 = pool.stats()
    # the timed region: K whole steps, nothing but the library's own work on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(wl, k, B)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st1 = pool.stats()
    # the same K steps once more with a HIP event before and after every kernel (per-kernel durations for the
    # roofline); the events cost about 0.1 ms per step, which is why the throughput is timed without them
    B.racer_prof_enable(pool.h, 1)
    B.racer_prof_read(pool.h)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(wl, k, B)
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t0
    prof = B.racer_prof_read(pool.h)
    B.racer_prof_enable(pool.h, 0)
    if args.copy_calib_mb:
        src = torch.empty(args.copy_calib_mb << 20, dtype=torch.uint8, device=Hn.DEV)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_per_step = dt * 1e3 / args.steps
    N, d, L, H = wl["N"], c["d"], c["L"], c["H"]
    lens = wl["lens"].astype(np.float64)
    pairs = float((lens * (lens + 1) / 2).sum())             # causal (query, key) pairs per layer
    attn_flop = 4.0 * d * pairs                                # 2*d_h for QK^T + 2*d_h for PV, per head, H heads
    attn_ms = prof["attention"][0] / max(prof["attention"][1], 1)
    attn_tflops = attn_flop / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0
    R = d * wl["esz"]
    lookups = st1["lookups"] - st0["lookups"]
    hits = st1["hits"] - st0["hits"]
    ways = pool.stats()["pages_emb"] / (wl["n_pages"] / 32)
    gather_bytes = N * (8 + 4 * ways + 4 + R + R)             # id + tag line + stamp + row read + row write
    gather_ms = prof["emb_gather"][0] / max(prof["emb_gather"][1], 1)
    gather_gbs = gather_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    useful_bytes = N * (8 + R + R)                             # without the tag line and the stamp
    useful_gbs = useful_bytes / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    kernels = {k: {"ms_per_launch": (v[0] / v[1] if v[1] else 0.0), "launches_per_step": v[1] / args.steps}
               for k, v in prof.items()}
    traffic, traffic_source = measured_traffic("attention_bf16_mfma", args.config) if c["bf16"] else (None, None)
    result = {
        "metric": "hstu_step_tokens_per_s", "value": N / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if c["bf16"] else "f32", "data": "synthetic",
        "ms_per_step_with_kernel_events": dt_events * 1e3 / args.steps,
        "passes": {"throughput": "K steps as the library runs them (a batch of this size: three pipelines on three "
                                 "streams)" if not args.one_pipeline else "K steps, one pipeline, kernel events on",
                   "kernels": "the same K steps again as one pipeline with a HIP event before and after every kernel"},
        "config": {"workload": c["desc"], "new_tokens_per_step": int(N), "requests": int(c["batch"]),
                   "emb_frac": c["alpha"], "causal_pairs_per_layer": pairs},
        "emb_gather": {"GBps": gather_gbs, "frac_of_hbm_peak": gather_gbs / PEAK_HBM_GBS,
                       "bytes_per_launch": gather_bytes, "ms_per_launch": gather_ms,
                       "useful_GBps": useful_gbs, "useful_bytes_per_launch": useful_bytes,
                       "hit_rate": hits / max(lookups, 1),
                       "note": "effective rate: this batch's traffic largely stays in the Infinity Cache and L2 "
                               "(four id batches in rotation); emb_gather_hbm is the HBM figure"},
        "roofline": {"kernel": "attention_bf16_mfma" if c["bf16"] else "attention_f32", "bound": "mfma",
                     "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / PEAK_BF16_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "flop_per_launch": attn_flop, "ms_per_launch": attn_ms},
        "kernels": kernels,
    }
    if not args.no_cpu:
        budget = args.cpu_tokens or (1024 if args.config == "tiny" else 24000)
        cb, take, ref = cpu_baseline(c, wl, synth, budget)
        result["cpu_baseline"] = cb
        # the oracle's outputs for its sample are compared with the GPU's for the same requests (same ids:
        # the first id set), with the measures of the parity tests
        from tests import parity
        one_step(wl, 0, B)
        torch.cuda.synchronize()
        got = wl["out"].float().cpu().numpy()
        rows = np.concatenate([np.arange(wl["reqs"][r][4], wl["reqs"][r][4] + int(wl["lens"][r])) for r in take])
        result["parity_max_rel_err"] = float(parity.rel_error_rows(got[rows], ref).max())
        result["parity"] = {"measure": "max over rows of max_i|gpu-ref| / max_i|ref|, fp64 oracle",
                            "rows": int(len(rows)), "requests": len(take),
                            "row_norm": result["parity_max_rel_err"],
                            "elementwise_floor_1e-2": float(parity.rel_error_elem(got[rows], ref).max()),
                            "tolerance_row_norm": parity.TOL_ROW[bool(c["bf16"])]}
    wl["model"].close()
    pool.close()
    if args.config == "mid" and not args.no_embheavy:
        # The Mid batch's gather is served largely from the caches (the figure above is an effective rate).  The gather
        # against HBM proper is the EMB-heavy configuration (2.1 M pooled lookups spread over a 40 GiB hot cache),
        # lookups only, timed here too so that the line carries it.
        del wl, pool
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        eh = emb_only_measure(args, CONFIGS["embheavy"], torch, Hn, B, synth, steps=min(args.steps, 20))
        result["emb_gather_hbm"] = {"workload": CONFIGS["embheavy"]["desc"], "GBps": eh["roofline"]["achieved"],
                                    "frac_of_hbm_peak": eh["roofline"]["frac"],
                                    "bytes_per_launch": eh["roofline"]["bytes_per_launch"],
                                    "ms_per_launch": eh["roofline"]["ms_per_launch"],
                                    "hit_rate": eh["config"]["hit_rate"], "lookups_per_launch": eh["config"]["lookups_per_step"],
                                    "ms_per_emb_lookup_call": eh["ms_per_step"],
                                    "useful_GBps": eh["roofline"]["useful_GBps"],
                                    "practical_ceiling_GBps": 5000.0,
                                    "frac_of_practical_ceiling": eh["roofline"]["achieved"] / 5000.0,
                                    "practical_ceiling_source": "profiles/hbm_ceilings.txt: random rows of a 40 GiB region "
                                                                "read and written out (bench.py --config hbmceiling)"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
