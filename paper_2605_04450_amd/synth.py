"""Seeded synthetic workloads shared by the oracle-side and GPU-side tests and the benchmark.

Nothing here is part of the method: no cache policy, no hashing into sets, no
HSTU arithmetic.  It only draws inputs with the shapes and skews the paper's
evaluation describes (Sec. V-A: Zipfian item popularity, 5K-15K-token user
profiles, user-specific histories) as stand-ins for its datasets and traces,
which are not redistributable.  Outputs are numpy arrays; both sides receive
the very same buffers.
"""
import math

import numpy as np

SEED_BASE = 20260504


def rng_for(config_index, stream=0):
    return np.random.default_rng([SEED_BASE + int(config_index), int(stream)])


# ---------------------------------------------------------------------------
# bounded Zipf ranks, P(k) ~ k^-s on 1..n, any s > 0 (rejection-inversion,
# Hoermann & Derflinger 1996: invert the integral of the continuous envelope
# x^-s, round to the nearest integer, accept with a squeeze/hat test)
# ---------------------------------------------------------------------------
def _H(x, s):
    if abs(s - 1.0) < 1e-12:
        return np.log(x)
    return np.expm1((1.0 - s) * np.log(x)) / (1.0 - s)


def _H_inv(y, s):
    if abs(s - 1.0) < 1e-12:
        return np.exp(y)
    t = np.maximum(y * (1.0 - s), -1.0 + 1e-300)
    return np.exp(np.log1p(t) / (1.0 - s))


def zipf_ranks(rng, n, s, size):
    """`size` ranks in 1..n with P(k) proportional to k**-s."""
    n = int(n)
    if n == 1:
        return np.ones(size, dtype=np.int64)
    h_x1 = _H(1.5, s) - 1.0
    h_n = _H(n + 0.5, s)
    thresh = 2.0 - _H_inv(_H(2.5, s) - 2.0 ** (-s), s)
    out = np.empty(size, dtype=np.int64)
    filled = 0
    while filled < size:
        m = max(1024, int((size - filled) * 1.3))
        u = h_n + rng.random(m) * (h_x1 - h_n)
        x = _H_inv(u, s)
        k = np.clip(np.rint(x), 1, n)
        ok = (k - x <= thresh) | (u >= _H(k + 0.5, s) - np.exp(-s * np.log(k)))
        k = k[ok].astype(np.int64)
        take = min(k.size, size - filled)
        out[filled:filled + take] = k[:take]
        filled += take
    return out


def _coprime_multiplier(n):
    a = max(3, int(n * 0.6180339887) | 1)
    while math.gcd(a, n) != 1:
        a += 2
    return a


def ranks_to_rows(ranks, n_rows, offset=12345):
    """Fixed bijection rank -> row id so hot rows scatter over the table."""
    a = _coprime_multiplier(n_rows)
    r = (np.asarray(ranks, dtype=np.int64) - 1) % n_rows
    # (r * a + offset) mod n without overflow: n_rows < 2**31 in every config here
    return ((r * a + offset) % n_rows).astype(np.int64)


def zipf_ids(rng, n_rows, s, size):
    return ranks_to_rows(zipf_ranks(rng, n_rows, s, size), n_rows)


def multi_feature_ids(rng, n_rows, n_features, s, n_tokens):
    """[n_tokens][n_features] ids; feature f draws from its own disjoint row range."""
    per = n_rows // n_features
    cols = [zipf_ids(rng, per, s, n_tokens) + f * per for f in range(n_features)]
    return np.stack(cols, axis=1).reshape(-1)


# ---------------------------------------------------------------------------
# history lengths and timestamps
# ---------------------------------------------------------------------------
def history_lengths(rng, batch, mean, lo, hi, sigma=0.6):
    """Lognormal lengths with the given arithmetic mean (before clipping)."""
    mu = math.log(mean) - 0.5 * sigma * sigma
    v = np.exp(rng.normal(mu, sigma, size=batch))
    return np.clip(np.rint(v), lo, hi).astype(np.int64)


def timestamps(rng, length, median_gap=60.0, sigma=1.5, start=1_600_000_000):
    """Non-decreasing int64 seconds: cumulative lognormal gaps."""
    gaps = np.exp(rng.normal(math.log(median_gap), sigma, size=length))
    return (start + np.cumsum(np.floor(gaps).astype(np.int64))).astype(np.int64)


# ---------------------------------------------------------------------------
# representable values
# ---------------------------------------------------------------------------
def to_bf16_bits(a):
    """fp32 array -> uint16 bf16 bit patterns (round to nearest even; inputs finite)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    return r.astype(np.uint16)


def from_bf16_bits(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def as_bf16_values(a):
    """fp32 array whose values are exactly representable in bf16."""
    return from_bf16_bits(to_bf16_bits(a))


_MIX_A, _MIX_B = 0xBF58476D1CE4E5B9, 0x94D049BB133111EB
_KEEP, _EXPO = 0x80FF80FF80FF80FF, 0x3E003E003E003E00


def _seed_word(seed):
    return (int(seed) * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF


def fill_table_bf16(dst_u16, seed, row_start=0, chunk_rows=1 << 18):
    """Fill a [rows][d] uint16 numpy array in place with finite bf16 bit patterns, |v| in [1/8, 1/2).

    Counter-based: one 64-bit integer mix per four elements, a pure function of
    (seed, row, column), so any block can be regenerated anywhere.  Rows are
    distinct with overwhelming probability.
    """
    rows, d = dst_u16.shape
    assert d % 4 == 0 and dst_u16.flags.c_contiguous
    w = d // 4
    flat = dst_u16.reshape(-1).view(np.uint64).reshape(rows, w)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        idx = (np.arange(r0 + row_start, r1 + row_start, dtype=np.uint64)[:, None] * np.uint64(w)
               + np.arange(w, dtype=np.uint64)[None, :])
        z = idx + np.uint64(_seed_word(seed))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MIX_A)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MIX_B)
        z = z ^ (z >> np.uint64(31))
        flat[r0:r1] = (z & np.uint64(_KEEP)) | np.uint64(_EXPO)
    return dst_u16


def fill_table_bf16_torch(dst_i16, seed, device, row_start=0, chunk_rows=1 << 21):
    """Same bits as fill_table_bf16, computed with torch integer ops on `device` and copied into
    the (possibly pinned) int16 host tensor `dst_i16` [rows][d].  For multi-GB tables."""
    import torch

    def s64(v):  # two's-complement view of a 64-bit constant
        return v - (1 << 64) if v >= (1 << 63) else v

    rows, d = dst_i16.shape
    w = d // 4
    flat = dst_i16.view(torch.int64).view(rows, w)
    cols = torch.arange(w, dtype=torch.int64, device=device)[None, :]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        z = torch.arange(r0 + row_start, r1 + row_start, dtype=torch.int64, device=device)[:, None] * w + cols
        z = z + s64(_seed_word(seed))
        z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * s64(_MIX_A)
        z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * s64(_MIX_B)
        z = z ^ ((z >> 31) & ((1 << 33) - 1))
        z = (z & s64(_KEEP)) | _EXPO
        flat[r0:r1].copy_(z)
    return dst_i16


def make_table(rng, rows, d, bf16):
    """Small tables for tests: N(0,1) values; bf16 tables come back as uint16 bit patterns."""
    t = rng.standard_normal((rows, d), dtype=np.float32)
    return to_bf16_bits(t) if bf16 else t


# ---------------------------------------------------------------------------
# model weights and cached KV
# ---------------------------------------------------------------------------
def make_weights(rng, L, d, H, n_pos, n_time, bf16):
    """Random-init HSTU weights (fp32 arrays; W1/W2 representable in bf16 when bf16=True)."""
    w = {
        "ln1_g": 1.0 + 0.05 * rng.standard_normal((L, d)),
        "ln1_b": 0.05 * rng.standard_normal((L, d)),
        "w1": rng.standard_normal((L, d, 4 * d)) / math.sqrt(d),
        "b1": 0.05 * rng.standard_normal((L, 4 * d)),
        "ln2_g": 1.0 + 0.05 * rng.standard_normal((L, d)),
        "ln2_b": 0.05 * rng.standard_normal((L, d)),
        "w2": rng.standard_normal((L, d, d)) / math.sqrt(d),
        "b2": 0.05 * rng.standard_normal((L, d)),
        "pos": 0.1 * rng.standard_normal((L, H, n_pos)),
        "time": 0.1 * rng.standard_normal((L, H, n_time)),
    }
    w = {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in w.items()}
    if bf16:
        for k in ("w1", "w2"):
            w[k] = as_bf16_values(w[k])
    return w


def make_requests(prefix_lens, new_lens, page_tokens):
    """Lay requests out back to back: returns (reqs, n_page_entries, n_ts, n_rows).

    reqs: list of (prefix_len, new_len, page_table_off, ts_off, x_off).
    """
    reqs, pto, tso, xo = [], 0, 0, 0
    for p, t in zip(prefix_lens, new_lens):
        p, t = int(p), int(t)
        reqs.append((p, t, pto, tso, xo))
        pto += (p + t + page_tokens - 1) // page_tokens
        tso += p + t
        xo += t
    return reqs, pto, tso, xo
