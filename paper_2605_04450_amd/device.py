"""Device-side conveniences over the binding: a pool and a model on cuda:0 whose memory PyTorch
allocates, and readers/writers of the KV page layout.  No arithmetic of the method lives here;
everything is computed by the C-ABI library."""
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
    """Device output -> numpy: fp32 values, or uint16 holding bf16 bit patterns."""
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
