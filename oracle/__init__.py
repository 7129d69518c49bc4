"""ctypes front end of the CPU oracle (test infrastructure, never the product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It loads ``liboracle.so`` built from the two C files beside it and
does nothing but marshal numpy arrays.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ["pool_oracle.c", "hstu_oracle.c"]

OK, DEFERRED, NOT_FOUND = 0, 1, 2
EINVAL, ENOMEM, ERANGE, EBUSY = -22, -12, -34, -16
TAG_EMPTY = 0xFFFFFFFF


def build(force=False):
    """Compile the oracle with gcc (no fast-math: the pooled fp32 sum is order-exact)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(s) for s in srcs + [os.path.join(_HERE, "racer_oracle.h")])
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB_PATH] + srcs + ["-lm"]
    subprocess.check_call(cmd)
    return _LIB_PATH


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "lookups", "hits", "misses", "unique_misses", "inserted", "evicted", "bypassed",
        "invalid_ids", "shrink_evicted", "shrink_moved", "pages_total", "pages_emb",
        "pages_kv_used", "pages_kv_free", "seqs_resident", "seqs_evicted", "batch")]

    def asdict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class HstuCfg(C.Structure):
    _fields_ = [("L", C.c_uint32), ("d", C.c_uint32), ("H", C.c_uint32),
                ("page_tokens", C.c_uint32), ("n_pos", C.c_uint32), ("n_time", C.c_uint32),
                ("n_scale", C.c_double), ("eps", C.c_double), ("store_bf16", C.c_int)]


class HstuReq(C.Structure):
    _fields_ = [("prefix_len", C.c_uint32), ("new_len", C.c_uint32),
                ("page_table_off", C.c_uint64), ("ts_off", C.c_uint64), ("x_off", C.c_uint64)]


class HstuWeights(C.Structure):
    _fields_ = [(n, C.POINTER(C.c_float)) for n in (
        "ln1_g", "ln1_b", "w1", "b1", "ln2_g", "ln2_b", "w2", "b2", "pos", "time")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = C.CDLL(_LIB_PATH)
        vp, u64, u32, i32, dbl = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int, C.c_double
        L.orc_pool_create.restype = vp
        L.orc_pool_create.argtypes = [u64, u32, u32, u32, dbl]
        L.orc_pool_destroy.argtypes = [vp]
        L.orc_pool_destroy.restype = None
        L.orc_pool_set_split.argtypes = [vp, dbl, C.POINTER(dbl)]
        L.orc_pool_stats.argtypes = [vp, C.POINTER(Stats)]
        L.orc_pool_num_sets.argtypes = [vp]
        L.orc_pool_num_sets.restype = u64
        L.orc_pool_ways.argtypes = [vp, u64]
        L.orc_pool_ways.restype = u32
        L.orc_pool_dump.argtypes = [vp, vp, vp, vp, vp]
        L.orc_pool_slot_of.argtypes = [vp, u64, u32]
        L.orc_pool_slot_of.restype = C.c_int64
        L.orc_kv_seq_reserve.argtypes = [vp, u64, u32, vp, u32, C.POINTER(u32)]
        L.orc_kv_seq_lookup.argtypes = [vp, u64, C.POINTER(u32), vp, u32, C.POINTER(u32)]
        for f in (L.orc_kv_seq_pin, L.orc_kv_seq_unpin, L.orc_kv_seq_release):
            f.argtypes = [vp, u64]
        L.orc_emb_set_of.argtypes = [vp, C.c_int64]
        L.orc_emb_set_of.restype = u64
        L.orc_emb_lookup.argtypes = [vp, vp, u64, u32, vp, u64, u32, i32, vp, vp]
        L.orc_emb_refill.argtypes = [vp, vp, u64, u64, vp]
        L.orc_emb_refill.restype = i32
        L.orc_round_bf16.argtypes = [C.c_float]
        L.orc_round_bf16.restype = C.c_float
        L.orc_f32_to_bf16_bits.argtypes = [C.c_float]
        L.orc_f32_to_bf16_bits.restype = C.c_uint16
        L.orc_bf16_bits_to_f32.argtypes = [C.c_uint16]
        L.orc_bf16_bits_to_f32.restype = C.c_float
        L.orc_silu.argtypes = [dbl]
        L.orc_silu.restype = dbl
        L.orc_time_bucket.argtypes = [C.c_int64, u32]
        L.orc_time_bucket.restype = u32
        L.orc_layernorm.argtypes = [vp, vp, vp, u32, dbl, vp]
        L.orc_layernorm.restype = None
        L.orc_attn_paged.argtypes = [C.POINTER(HstuCfg), u32, vp, vp, u32, u32, vp, vp, vp, vp, vp]
        L.orc_attn_paged.restype = None
        L.orc_hstu_step.argtypes = [C.POINTER(HstuCfg), C.POINTER(HstuWeights), C.POINTER(HstuReq),
                                    u32, vp, vp, u64, vp, vp, vp, i32]
        L.orc_kv_elems_per_page.argtypes = [C.POINTER(HstuCfg)]
        L.orc_kv_elems_per_page.restype = u64
        L.orc_kv_offset.argtypes = [C.POINTER(HstuCfg), u64, u32, u32, u32, u32]
        L.orc_kv_offset.restype = u64
        L.orc_max_threads.restype = i32
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class Pool:
    """Host simulator of the shared page pool, its KV sequence table and the EMB cache."""

    def __init__(self, n_pages, page_tokens, slots_per_page, w_max=32, emb_frac0=0.5):
        self._h = lib().orc_pool_create(n_pages, page_tokens, slots_per_page, w_max, float(emb_frac0))
        if not self._h:
            raise ValueError("orc_pool_create rejected the geometry")
        self.n_pages, self.page_tokens, self.spp, self.w_max = n_pages, page_tokens, slots_per_page, w_max

    def close(self):
        if self._h:
            lib().orc_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    @property
    def num_sets(self):
        return int(lib().orc_pool_num_sets(self._h))

    def ways(self, s):
        return int(lib().orc_pool_ways(self._h, s))

    def set_of(self, id_):
        return int(lib().orc_emb_set_of(self._h, int(id_)))

    def slot_of(self, s, w):
        return int(lib().orc_pool_slot_of(self._h, s, w))

    def set_split(self, emb_frac):
        ach = C.c_double(0.0)
        rc = lib().orc_pool_set_split(self._h, float(emb_frac), C.byref(ach))
        return rc, ach.value

    def stats(self):
        st = Stats()
        lib().orc_pool_stats(self._h, C.byref(st))
        return st.asdict()

    def dump(self):
        st = self.stats()
        emb_pages = np.zeros(st["pages_emb"], dtype=np.int64)
        owner = np.zeros(self.n_pages, dtype=np.uint8)
        S = self.num_sets
        tags = np.zeros((S, self.w_max), dtype=np.uint32)
        stamps = np.zeros((S, self.w_max), dtype=np.uint32)
        lib().orc_pool_dump(self._h, _ptr(emb_pages), _ptr(owner), _ptr(tags), _ptr(stamps))
        return {"emb_pages": emb_pages, "owner": owner, "tags": tags, "stamps": stamps}

    def kv_reserve(self, key, tokens):
        cap = (max(tokens, 1) + self.page_tokens - 1) // self.page_tokens + 8
        n = C.c_uint32(0)
        # a sequence may already hold more pages than `tokens` needs: ask for the count first
        lib().orc_kv_seq_lookup(self._h, key, None, None, 0, C.byref(n))
        cap = max(cap, n.value)
        pages = np.zeros(cap, dtype=np.int32)
        rc = lib().orc_kv_seq_reserve(self._h, key, tokens, _ptr(pages), cap, C.byref(n))
        return rc, pages[: n.value].copy() if rc == OK else None

    def kv_lookup(self, key):
        n, tok = C.c_uint32(0), C.c_uint32(0)
        rc = lib().orc_kv_seq_lookup(self._h, key, C.byref(tok), None, 0, C.byref(n))
        if rc != OK:
            return rc, 0, None
        pages = np.zeros(n.value, dtype=np.int32)
        lib().orc_kv_seq_lookup(self._h, key, C.byref(tok), _ptr(pages), n.value, C.byref(n))
        return OK, tok.value, pages

    def kv_pin(self, key):
        return lib().orc_kv_seq_pin(self._h, key)

    def kv_unpin(self, key):
        return lib().orc_kv_seq_unpin(self._h, key)

    def kv_release(self, key):
        return lib().orc_kv_seq_release(self._h, key)

    def emb_lookup(self, ids, table, bag=1, want_out=True):
        """table: [rows][d] float32, or uint16 holding bf16 bit patterns; with want_out=False it may be
        just (rows, d, dtype), since no row is read then. Returns (rc, out, hit)."""
        ids = _c(ids, np.int64)
        n = ids.size
        if isinstance(table, tuple):
            assert not want_out
            rows, d, dtype = table
            table = None
        else:
            assert table.dtype in (np.float32, np.uint16) and table.ndim == 2 and table.flags.c_contiguous
            rows, d, dtype = table.shape[0], table.shape[1], table.dtype
        elem = 0 if dtype == np.float32 else 1
        out = np.zeros((n // bag if bag else 0, d), dtype=dtype) if want_out else None
        hit = np.zeros(n, dtype=np.uint8)
        rc = lib().orc_emb_lookup(self._h, _ptr(ids), n, bag, _ptr(table), rows, d, elem, _ptr(out), _ptr(hit))
        return rc, out, hit

    def emb_refill(self, ids, rows):
        """Fill empty ways with `ids` (hottest first). Returns (rc, rows inserted)."""
        ids = _c(ids, np.int64)
        ins = C.c_uint64(0)
        rc = lib().orc_emb_refill(self._h, _ptr(ids), ids.size, rows, C.byref(ins))
        return rc, int(ins.value)


def round_bf16(a):
    """Round a float array to bf16 (nearest even) with the oracle's own routine, return fp32."""
    a = np.asarray(a, dtype=np.float32)
    f = np.vectorize(lambda v: lib().orc_round_bf16(float(v)), otypes=[np.float32])
    return f(a) if a.size else a.copy()


def silu(x):
    return lib().orc_silu(float(x))


def time_bucket(dt, n_time):
    return int(lib().orc_time_bucket(int(dt), n_time))


def layernorm(x, g, b, eps):
    x = _c(x, np.float64)
    g = _c(g, np.float32)
    b = _c(b, np.float32)
    y = np.zeros_like(x)
    lib().orc_layernorm(_ptr(x), _ptr(g), _ptr(b), x.size, float(eps), _ptr(y))
    return y


def make_cfg(L, d, H, page_tokens, n_pos, n_time, n_scale, eps=1e-6, store_bf16=False):
    return HstuCfg(L, d, H, page_tokens, n_pos, n_time, float(n_scale), float(eps), int(bool(store_bf16)))


def kv_elems_per_page(cfg):
    return int(lib().orc_kv_elems_per_page(C.byref(cfg)))


def kv_offset(cfg, page, layer, kv, head, tok):
    return int(lib().orc_kv_offset(C.byref(cfg), page, layer, kv, head, tok))


def attn_paged(cfg, layer, pos, time, P, T, pages, ts, kv_mem, q):
    """One layer's attention for one request; q [T][d] fp64 -> o [T][d] fp64."""
    pos = _c(pos, np.float32)
    time = _c(time, np.float32)
    pages = _c(pages, np.int32)
    ts = _c(ts, np.int64)
    q = _c(q, np.float64)
    assert kv_mem.dtype == np.float32 and kv_mem.flags.c_contiguous
    o = np.zeros((T, cfg.d), dtype=np.float64)
    lib().orc_attn_paged(C.byref(cfg), layer, _ptr(pos), _ptr(time), P, T, _ptr(pages), _ptr(ts),
                         _ptr(kv_mem), _ptr(q), _ptr(o))
    return o


_W_NAMES = ("ln1_g", "ln1_b", "w1", "b1", "ln2_g", "ln2_b", "w2", "b2", "pos", "time")


def hstu_step(cfg, weights, reqs, page_tables, kv_mem, x_in, ts, threads=0):
    """weights: dict name -> fp32 array (all layers). reqs: list of
    (prefix_len, new_len, page_table_off, ts_off, x_off). kv_mem: fp32 array of
    whole pages, updated in place. Returns (rc, out [N][d] fp64)."""
    keep = {n: _c(weights[n], np.float32) for n in _W_NAMES}
    w = HstuWeights(*[keep[n].ctypes.data_as(C.POINTER(C.c_float)) for n in _W_NAMES])
    arr = (HstuReq * max(len(reqs), 1))()
    for i, r in enumerate(reqs):
        arr[i] = HstuReq(*[int(v) for v in r])
    page_tables = _c(page_tables, np.int32)
    x_in = _c(x_in, np.float32)
    ts = _c(ts, np.int64)
    assert kv_mem.dtype == np.float32 and kv_mem.flags.c_contiguous
    per_page = kv_elems_per_page(cfg)
    assert kv_mem.size % per_page == 0
    out = np.zeros((x_in.shape[0], cfg.d), dtype=np.float64)
    rc = lib().orc_hstu_step(C.byref(cfg), C.byref(w), arr, len(reqs), _ptr(page_tables), _ptr(kv_mem),
                             kv_mem.size // per_page, _ptr(x_in), _ptr(ts), _ptr(out), threads)
    return rc, out


def max_threads():
    return int(lib().orc_max_threads())
