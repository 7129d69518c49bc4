"""Thin ctypes binding of libracer_hip.so: same names as the C-ABI, argument marshalling only.

Tensors are torch tensors used as plain device (or pinned host) buffers; every step of the
path runs in the library's kernels.  There is no fallback: a missing library is an error.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libracer_hip.so")

OK, DEFERRED, NOT_FOUND = 0, 1, 2
EINVAL, ENOMEM, ERANGE, EBUSY, EHIP = -22, -12, -34, -16, -5
ELEM_F32, ELEM_BF16 = 0, 1
TAG_EMPTY = 0xFFFFFFFF

EXPORTS = [
    "pool_create", "pool_destroy", "pool_set_split", "pool_reserve", "pool_stats", "pool_dump", "emb_cache_dump",
    "pool_num_sets", "pool_slot_of", "kv_seq_reserve", "kv_seq_lookup", "kv_seq_pin", "kv_seq_unpin",
    "kv_seq_release", "emb_lookup", "emb_lookup_noalloc", "emb_refill", "pool_add_table", "emb_lookup_tables", "hstu_model_create", "hstu_model_destroy", "hstu_step",
    "hstu_attn_paged", "racer_last_error", "racer_prof_enable", "racer_prof_read",
    "alpha_ctl_create", "alpha_ctl_destroy", "alpha_ctl_decide", "alpha_ctl_reward", "racer_hbm_probe",
]
PROF_KINDS = ("emb_gather", "emb_miss", "layernorm", "gemm_front", "attention", "gemm_back", "attn_reduce")


class Prof(C.Structure):
    _fields_ = [("ms", C.c_double * 7), ("launches", C.c_uint64 * 7)]


class PoolCfg(C.Structure):
    _fields_ = [("row_bytes", C.c_uint32), ("elem", C.c_uint32), ("page_tokens", C.c_uint32),
                ("w_max", C.c_uint32), ("host_table", C.c_void_p), ("rows", C.c_uint64),
                ("emb_frac0", C.c_double)]


class PoolStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "lookups", "hits", "misses", "unique_misses", "inserted", "evicted", "bypassed", "invalid_ids",
        "shrink_evicted", "shrink_moved", "pages_total", "pages_emb", "pages_kv_used", "pages_kv_free",
        "seqs_resident", "seqs_evicted", "batch", "bad_pages", "unordered_ts", "ws_allocs")]

    def asdict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class Reserve(C.Structure):
    _fields_ = [("max_lookups", C.c_uint64), ("max_requests", C.c_uint32), ("max_new_tokens", C.c_uint64),
                ("max_seq_tokens", C.c_uint32)]


class AlphaState(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("hot_user_ratio", "kv_hit_rate", "emb_hit_rate", "mean_seq_len",
                                          "slo_violation", "alpha", "p99_latency_ms")]


class HstuCfg(C.Structure):
    _fields_ = [("L", C.c_uint32), ("d", C.c_uint32), ("H", C.c_uint32), ("elem", C.c_uint32),
                ("page_tokens", C.c_uint32), ("n_pos", C.c_uint32), ("n_time", C.c_uint32),
                ("n_scale", C.c_float), ("eps", C.c_float)]


class HstuWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ln1_g", "ln1_b", "w1", "b1", "ln2_g", "ln2_b", "w2", "b2", "pos", "time")]


class HstuReq(C.Structure):
    _fields_ = [("prefix_len", C.c_uint32), ("new_len", C.c_uint32), ("page_table_off", C.c_uint64),
                ("ts_off", C.c_uint64), ("x_off", C.c_uint64)]


_lib = None


def load():
    """Open the library and declare the signatures; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libracer_hip.so is missing: run `python __graft_entry__.py` to build it "
                           "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, u64, u32, i32, dbl = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32, C.c_double
    L.pool_create.argtypes = [vp, u64, u64, C.POINTER(PoolCfg), C.POINTER(vp)]
    L.pool_destroy.argtypes = [vp]
    L.pool_set_split.argtypes = [vp, dbl, vp, C.POINTER(dbl)]
    L.pool_stats.argtypes = [vp, C.POINTER(PoolStats)]
    L.pool_dump.argtypes = [vp, vp, vp]
    L.emb_cache_dump.argtypes = [vp, vp, vp]
    L.pool_num_sets.argtypes = [vp]
    L.pool_num_sets.restype = u64
    L.pool_slot_of.argtypes = [vp, u64, u32]
    L.pool_slot_of.restype = C.c_int64
    L.kv_seq_reserve.argtypes = [vp, u64, u32, vp, u32, C.POINTER(u32)]
    L.kv_seq_lookup.argtypes = [vp, u64, C.POINTER(u32), vp, u32, C.POINTER(u32)]
    for f in (L.kv_seq_pin, L.kv_seq_unpin, L.kv_seq_release):
        f.argtypes = [vp, u64]
    L.pool_reserve.argtypes = [vp, vp, C.POINTER(Reserve), vp]
    L.alpha_ctl_create.argtypes = [C.c_double, C.POINTER(vp)]
    L.alpha_ctl_destroy.argtypes = [vp]
    L.alpha_ctl_decide.argtypes = [vp, C.POINTER(AlphaState), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    L.alpha_ctl_reward.argtypes = [C.c_double, C.c_double, C.c_double]
    L.alpha_ctl_reward.restype = C.c_double
    L.emb_lookup.argtypes = [vp, vp, u64, u32, vp, vp, vp]
    L.emb_lookup_noalloc.argtypes = [vp, vp, u64, u32, vp, vp, vp]
    L.emb_refill.argtypes = [vp, vp, u64, vp]
    L.pool_add_table.argtypes = [vp, vp, u64, u32, C.POINTER(u32)]
    L.emb_lookup_tables.argtypes = [vp, vp, vp, u64, u32, vp, vp, vp]
    L.hstu_model_create.argtypes = [C.POINTER(HstuCfg), C.POINTER(HstuWeights), C.POINTER(vp)]
    L.hstu_model_destroy.argtypes = [vp]
    L.hstu_step.argtypes = [vp, vp, C.POINTER(HstuReq), u32, vp, u64, vp, vp, vp, vp]
    L.hstu_attn_paged.argtypes = [vp, vp, u32, C.POINTER(HstuReq), u32, vp, u64, vp, vp, vp, vp]
    L.racer_hbm_probe.argtypes = [vp, u64, u32, u64, vp, u64, vp]
    L.racer_prof_enable.argtypes = [vp, i32]
    L.racer_prof_read.argtypes = [vp, C.POINTER(Prof)]
    L.racer_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("pool_num_sets", "pool_slot_of", "racer_last_error", "alpha_ctl_reward"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def racer_hbm_probe(region, row_bytes, n_reads, out=None, seed=1, stream=None):
    """Random row reads out of the device tensor `region` (measurement aid)."""
    return load().racer_hbm_probe(_dp(region), region.numel() * region.element_size(), row_bytes, n_reads, _dp(out), seed,
                                  _stream_ptr(stream))


def last_error():
    return load().racer_last_error().decode()


def racer_prof_enable(pool, on):
    return load().racer_prof_enable(pool, int(on))


def racer_prof_read(pool):
    """{kind: (total ms, launches)} of the intervals recorded since the last read."""
    pr = Prof()
    rc = load().racer_prof_read(pool, C.byref(pr))
    if rc != OK:
        raise RuntimeError("racer_prof_read failed: %d %s" % (rc, last_error()))
    return {k: (pr.ms[i], int(pr.launches[i])) for i, k in enumerate(PROF_KINDS)}


def _dp(t):
    """Device (or host) address of a torch tensor / numpy array, None -> NULL."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data_as(C.c_void_p)
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def pool_create(dev_base, nbytes, page_size, row_bytes, elem, page_tokens, w_max=32, host_table=None, rows=0,
                emb_frac0=0.5):
    """dev_base: torch uint8 device tensor backing the pool, or None for a metadata-only pool.
    host_table: pinned torch tensor [rows][d] (or None).  Returns (rc, handle)."""
    cfg = PoolCfg(row_bytes, elem, page_tokens, w_max, _dp(host_table), rows, float(emb_frac0))
    h = C.c_void_p()
    rc = load().pool_create(_dp(dev_base), nbytes, page_size, C.byref(cfg), C.byref(h))
    return rc, (h if rc == OK else None)


def pool_destroy(pool):
    return load().pool_destroy(pool)


def pool_set_split(pool, emb_frac, stream=None, device=True):
    ach = C.c_double(0.0)
    rc = load().pool_set_split(pool, float(emb_frac), _stream_ptr(stream) if device else None, C.byref(ach))
    return rc, ach.value


def pool_reserve(pool, model, max_lookups=0, max_requests=0, max_new_tokens=0, max_seq_tokens=0, stream=None):
    """Size the library's work spaces ahead of time (model: handle or None)."""
    r = Reserve(max_lookups, max_requests, max_new_tokens, max_seq_tokens)
    return load().pool_reserve(pool, model, C.byref(r), _stream_ptr(stream))


class AlphaController:
    """The split controller: decide(...) -> (step, next fraction, burst flag)."""

    def __init__(self, slo_ms):
        self.h = C.c_void_p()
        rc = load().alpha_ctl_create(float(slo_ms), C.byref(self.h))
        if rc != OK:
            raise ValueError("alpha_ctl_create failed: %d" % rc)

    def decide(self, alpha, p99_latency_ms, hot_user_ratio=0.0, kv_hit_rate=0.0, emb_hit_rate=0.0, mean_seq_len=0.0,
               slo_violation=0.0):
        s = AlphaState(hot_user_ratio, kv_hit_rate, emb_hit_rate, mean_seq_len, slo_violation, alpha, p99_latency_ms)
        step, nxt, burst = C.c_double(0.0), C.c_double(0.0), C.c_int32(0)
        rc = load().alpha_ctl_decide(self.h, C.byref(s), C.byref(step), C.byref(nxt), C.byref(burst))
        if rc != OK:
            raise ValueError("alpha_ctl_decide failed: %d" % rc)
        return step.value, nxt.value, bool(burst.value)

    def close(self):
        if self.h:
            load().alpha_ctl_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def alpha_reward(slo_satisfaction, p99_latency_ms, slo_ms):
    return load().alpha_ctl_reward(float(slo_satisfaction), float(p99_latency_ms), float(slo_ms))


def pool_stats(pool):
    st = PoolStats()
    rc = load().pool_stats(pool, C.byref(st))
    if rc != OK:
        raise RuntimeError("pool_stats failed: %d %s" % (rc, last_error()))
    return st.asdict()


def pool_num_sets(pool):
    return int(load().pool_num_sets(pool))


def pool_slot_of(pool, s, w):
    return int(load().pool_slot_of(pool, s, w))


def pool_dump(pool):
    st = pool_stats(pool)
    emb_pages = np.zeros(st["pages_emb"], dtype=np.int64)
    owner = np.zeros(st["pages_total"], dtype=np.uint8)
    rc = load().pool_dump(pool, _dp(emb_pages), _dp(owner))
    assert rc == OK
    return {"emb_pages": emb_pages, "owner": owner}


def emb_cache_dump(pool, w_max):
    S = pool_num_sets(pool)
    tags = np.zeros((S, w_max), dtype=np.uint32)
    stamps = np.zeros((S, w_max), dtype=np.uint32)
    rc = load().emb_cache_dump(pool, _dp(tags), _dp(stamps))
    if rc != OK:
        raise RuntimeError("emb_cache_dump failed: %d %s" % (rc, last_error()))
    return tags, stamps


def kv_seq_reserve(pool, key, tokens, cap=None):
    n = C.c_uint32(0)
    load().kv_seq_lookup(pool, key, None, None, 0, C.byref(n))
    cap = max(cap or 0, n.value, tokens + 64)  # never fewer than one entry per token
    pages = np.zeros(cap, dtype=np.int32)
    rc = load().kv_seq_reserve(pool, key, tokens, _dp(pages), cap, C.byref(n))
    return rc, (pages[: n.value].copy() if rc == OK else None)


def kv_seq_lookup(pool, key):
    n, tok = C.c_uint32(0), C.c_uint32(0)
    rc = load().kv_seq_lookup(pool, key, C.byref(tok), None, 0, C.byref(n))
    if rc != OK:
        return rc, 0, None
    pages = np.zeros(max(n.value, 1), dtype=np.int32)
    load().kv_seq_lookup(pool, key, C.byref(tok), _dp(pages), n.value, C.byref(n))
    return OK, tok.value, pages[: n.value].copy()


def kv_seq_pin(pool, key):
    return load().kv_seq_pin(pool, key)


def kv_seq_unpin(pool, key):
    return load().kv_seq_unpin(pool, key)


def kv_seq_release(pool, key):
    return load().kv_seq_release(pool, key)


def emb_lookup(pool, ids, out, bag=1, hit_flags=None, stream=None):
    """ids: int64 device tensor [n]; out: device tensor [n/bag][d]; hit_flags: uint8 device tensor [n] or None."""
    return load().emb_lookup(pool, _dp(ids), ids.numel(), bag, _dp(out), _dp(hit_flags), _stream_ptr(stream))


NOALLOC_MAX_LOOKUPS = 16384
NOALLOC_MAX_ROW_BYTES_TOTAL = 8 << 20


def emb_lookup_noalloc(pool, ids, out, bag=1, hit_flags=None, stream=None):
    """emb_lookup that allocates nothing (fixed work space inside the library; see the header for its limits)."""
    return load().emb_lookup_noalloc(pool, _dp(ids), ids.numel(), bag, _dp(out), _dp(hit_flags), _stream_ptr(stream))


def pool_add_table(pool, host_table, rows, row_bytes):
    """host_table: pinned host tensor [rows][row_bytes / element size]. Returns (rc, table number)."""
    t = C.c_uint32(0)
    rc = load().pool_add_table(pool, _dp(host_table), rows, row_bytes, C.byref(t))
    return rc, t.value


def emb_lookup_tables(pool, table_of, ids, out, bag=1, hit_flags=None, stream=None):
    """table_of: int32/uint32 device tensor [n]; ids: int64 device tensor [n] (rows inside their tables)."""
    return load().emb_lookup_tables(pool, _dp(table_of), _dp(ids), ids.numel(), bag, _dp(out), _dp(hit_flags),
                                    _stream_ptr(stream))


def emb_refill(pool, ids, stream=None):
    """ids: int64 device tensor [n], hottest first."""
    return load().emb_refill(pool, _dp(ids), ids.numel(), _stream_ptr(stream))


def hstu_model_create(L, d, H, elem, page_tokens, n_pos, n_time, n_scale, eps, weights):
    """weights: dict name -> device tensor (kept alive by the caller). Returns (rc, handle)."""
    cfg = HstuCfg(L, d, H, elem, page_tokens, n_pos, n_time, float(n_scale), float(eps))
    w = HstuWeights(*[_dp(weights[n]) for n in ("ln1_g", "ln1_b", "w1", "b1", "ln2_g", "ln2_b", "w2", "b2", "pos", "time")])
    h = C.c_void_p()
    rc = load().hstu_model_create(C.byref(cfg), C.byref(w), C.byref(h))
    return rc, (h if rc == OK else None)


def hstu_model_destroy(model):
    return load().hstu_model_destroy(model)


def make_reqs(reqs):
    arr = (HstuReq * max(len(reqs), 1))()
    for i, r in enumerate(reqs):
        arr[i] = HstuReq(*[int(v) for v in r])
    return arr


def hstu_step(pool, model, reqs, kv_page_tables, x_in, ts, out, stream=None):
    """reqs: list of (prefix_len, new_len, page_table_off, ts_off, x_off) or a prepared HstuReq array
    with its length, given as (array, B)."""
    arr, B = reqs if isinstance(reqs, tuple) else (make_reqs(reqs), len(reqs))
    return load().hstu_step(pool, model, arr, B, _dp(kv_page_tables), kv_page_tables.numel(), _dp(x_in), _dp(ts),
                            _dp(out), _stream_ptr(stream))


def hstu_attn_paged(pool, model, layer, reqs, kv_page_tables, q, ts, o, stream=None):
    arr, B = reqs if isinstance(reqs, tuple) else (make_reqs(reqs), len(reqs))
    return load().hstu_attn_paged(pool, model, layer, arr, B, _dp(kv_page_tables), kv_page_tables.numel(), _dp(q),
                                  _dp(ts), _dp(o), _stream_ptr(stream))
