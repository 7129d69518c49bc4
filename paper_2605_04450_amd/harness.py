"""Glue used by the GPU tests, the smoke check and the benchmark: builds a pool and a model on
cuda:0 from synthetic inputs and runs the library on them.  No arithmetic of the method lives
here; everything is computed by the C-ABI library."""
import math

import numpy as np
import torch

from . import binding as B
from . import synth

DEV = "cuda:0"


def elem_size(elem):
    return 2 if elem == B.ELEM_BF16 else 4


def torch_dtype(elem):
    return torch.bfloat16 if elem == B.ELEM_BF16 else torch.float32


def to_device_table(table_np):
    """numpy table (fp32, or uint16 bf16 bits) -> pinned host tensor the kernels read over PCIe."""
    t = torch.from_numpy(table_np.view(np.int16) if table_np.dtype == np.uint16 else table_np)
    pinned = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    pinned.copy_(t)
    return pinned


class Pool:
    """A device pool with (optionally) a pinned host table behind its EMB side."""

    def __init__(self, n_pages, page_size, row_bytes, elem, page_tokens, w_max=32, table=None, emb_frac0=0.5,
                 zero_fill=False):
        self.n_pages, self.page_size, self.row_bytes, self.elem = n_pages, page_size, row_bytes, elem
        self.page_tokens, self.w_max = page_tokens, w_max
        nbytes = n_pages * page_size
        self.mem = (torch.zeros if zero_fill else torch.empty)(nbytes, dtype=torch.uint8, device=DEV)
        self.table = table  # pinned host tensor, kept alive here
        rows = table.shape[0] if table is not None else 0
        rc, self.h = B.pool_create(self.mem, nbytes, page_size, row_bytes, elem, page_tokens, w_max, table, rows,
                                   emb_frac0)
        if rc != B.OK:
            raise RuntimeError("pool_create failed: %d %s" % (rc, B.last_error()))

    def close(self):
        if self.h is not None:
            torch.cuda.synchronize()
            B.pool_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def lookup(self, ids_dev, bag=1, want_hits=True):
        n = ids_dev.numel()
        d = self.row_bytes // elem_size(self.elem)
        out = torch.empty((n // bag, d), dtype=torch_dtype(self.elem), device=DEV)
        hit = torch.empty(n, dtype=torch.uint8, device=DEV) if want_hits else None
        rc = B.emb_lookup(self.h, ids_dev, out, bag, hit)
        if rc != B.OK:
            raise RuntimeError("emb_lookup failed: %d %s" % (rc, B.last_error()))
        return out, hit

    def stats(self):
        return B.pool_stats(self.h)

    def cache_dump(self):
        return B.emb_cache_dump(self.h, self.w_max)

    def slot_rows(self, slots):
        """Rows stored at the given physical slot numbers (numpy uint8 [len][row_bytes])."""
        idx = torch.as_tensor(np.asarray(slots, dtype=np.int64), device=DEV)
        return self.mem.view(-1, self.row_bytes)[idx].cpu().numpy()


def out_to_numpy(out, elem):
    """Device output -> numpy in the oracle's convention (fp32, or uint16 bf16 bits)."""
    if elem == B.ELEM_BF16:
        return out.view(torch.int16).cpu().numpy().view(np.uint16)
    return out.cpu().numpy()


class Model:
    """HSTU weights on the device + the library's model handle."""

    def __init__(self, L, d, H, elem, page_tokens, n_pos, n_time, n_scale, weights_np, eps=1e-6):
        self.L, self.d, self.H, self.elem = L, d, H, elem
        self.page_tokens, self.n_pos, self.n_time, self.n_scale, self.eps = page_tokens, n_pos, n_time, n_scale, eps
        self.w = {}
        for k, v in weights_np.items():
            t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(DEV)
            if k in ("w1", "w2") and elem == B.ELEM_BF16:
                t = t.to(torch.bfloat16)  # values are already bf16-representable: exact
            self.w[k] = t.contiguous()
        rc, self.h = B.hstu_model_create(L, d, H, elem, page_tokens, n_pos, n_time, n_scale, eps, self.w)
        if rc != B.OK:
            raise RuntimeError("hstu_model_create failed: %d %s" % (rc, B.last_error()))

    def page_size(self):
        return self.page_tokens * 2 * self.L * self.d * elem_size(self.elem)

    def close(self):
        if self.h is not None:
            torch.cuda.synchronize()
            B.hstu_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kv_block_elem_offset(L, d, H, pt, page, layer, kv, head):
    """Element offset of the K (kv=0) or V (kv=1) block of (layer, head) in the device pool,
    counted in elements from the pool base: pages of [layer][K|V][head] blocks of pt*d_h elements."""
    dh = d // H
    return page * (pt * 2 * L * d) + (((layer * 2 + kv) * H + head) * pt * dh)


def write_prefix_kv(pool_mem_elems, L, d, H, pt, pages, k_rows, v_rows, layer):
    """Place cached prefix K,V ([P][d] tensors on the device, storage dtype) of one layer into the
    given pages in the library's layout: K blocks [token][d_h], V blocks [d_h][token]."""
    dh = d // H
    P = k_rows.shape[0]
    for pi, page in enumerate(pages):
        t0 = pi * pt
        if t0 >= P:
            break
        t1 = min(P, t0 + pt)
        for h in range(H):
            ko = kv_block_elem_offset(L, d, H, pt, int(page), layer, 0, h)
            vo = kv_block_elem_offset(L, d, H, pt, int(page), layer, 1, h)
            pool_mem_elems[ko:ko + (t1 - t0) * dh] = k_rows[t0:t1, h * dh:(h + 1) * dh].reshape(-1)
            vblk = pool_mem_elems[vo:vo + pt * dh].view(dh, pt)
            vblk[:, : t1 - t0] = v_rows[t0:t1, h * dh:(h + 1) * dh].t()


def read_kv(pool_mem_elems, L, d, H, pt, pages, S, layer):
    """Inverse of write_prefix_kv: K,V [S][d] of one layer gathered from the pages (device tensors)."""
    dh = d // H
    K = torch.empty((S, d), dtype=pool_mem_elems.dtype, device=pool_mem_elems.device)
    V = torch.empty_like(K)
    for pi, page in enumerate(pages):
        t0 = pi * pt
        if t0 >= S:
            break
        t1 = min(S, t0 + pt)
        for h in range(H):
            ko = kv_block_elem_offset(L, d, H, pt, int(page), layer, 0, h)
            vo = kv_block_elem_offset(L, d, H, pt, int(page), layer, 1, h)
            K[t0:t1, h * dh:(h + 1) * dh] = pool_mem_elems[ko:ko + (t1 - t0) * dh].view(t1 - t0, dh)
            V[t0:t1, h * dh:(h + 1) * dh] = pool_mem_elems[vo:vo + pt * dh].view(dh, pt)[:, : t1 - t0].t()
    return K, V


def rel_error_rows(got, ref):
    """Row-wise relative error in the max norm: max_i |got_i - ref_i| / max_i |ref_i| per row."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return num / den


def smoke_check():
    """One tiny serving step (EMB lookup then HSTU step) on cuda:0, checked against the oracle."""
    import oracle
    L, d, H, pt, rows = 1, 64, 2, 16, 5000
    rng = synth.rng_for(0, 99)
    table = synth.make_table(rng, rows, d, bf16=False)
    lens = [40, 17]
    reqs, n_pt, n_ts, N = synth.make_requests([0, 0], lens, pt)
    n_pos, n_time, n_scale = 64, 16, 64.0
    w = synth.make_weights(rng, L, d, H, n_pos, n_time, bf16=False)
    page_size = pt * 2 * L * d * 4
    n_pages = 64
    pool = Pool(n_pages, page_size, d * 4, B.ELEM_F32, pt, 32, to_device_table(table), 0.5)
    model = Model(L, d, H, B.ELEM_F32, pt, n_pos, n_time, n_scale, w)
    orc = oracle.Pool(n_pages, pt, page_size // (d * 4), 32, 0.5)
    ids = synth.zipf_ids(rng, rows, 1.0, N)
    for _ in range(2):
        x, hit = pool.lookup(torch.from_numpy(ids).to(DEV))
        rc, ox, ohit = orc.emb_lookup(ids, table)
        assert np.array_equal(hit.cpu().numpy(), ohit), "hit flags differ from the oracle"
        assert np.array_equal(x.cpu().numpy(), ox), "gathered rows differ from the oracle"
    pages = []
    for key, s in enumerate(lens):
        rc, pg = B.kv_seq_reserve(pool.h, key, s)
        assert rc == B.OK
        assert np.array_equal(pg, orc.kv_reserve(key, s)[1])
        pages.append(pg)
    pts = np.concatenate(pages).astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng, s) for s in lens])
    out = torch.empty((N, d), dtype=torch.float32, device=DEV)
    rc = B.hstu_step(pool.h, model.h, reqs, torch.from_numpy(pts).to(DEV), x, torch.from_numpy(ts).to(DEV), out)
    assert rc == B.OK, (rc, B.last_error())
    torch.cuda.synchronize()
    cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale, 1e-6, False)
    kv = np.zeros(n_pages * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    rc, ref = oracle.hstu_step(cfg, w, reqs, pts, kv, ox, ts)
    err = rel_error_rows(out.cpu().numpy(), ref).max()
    assert err < 1e-4, "hstu_step differs from the oracle: %g" % err
    assert pool.stats()["bad_pages"] == 0
    model.close()
    pool.close()
