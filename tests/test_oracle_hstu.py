"""Pins for the oracle's HSTU layer stack (CPU only).

The oracle is compared with library routines (torch fp64 layer_norm / silu /
matmul in a dense masked-matrix formulation, torch's bf16 conversion, Python's
int.bit_length), with the paper's KV-size figures, and with properties that
hold by construction of causal attention over a cache (prefix equivalence,
future-independence, page-table and page-size invariance, exact scaling).
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2605_04450_amd import synth
from tests.test_oracle_pool import golden


def build_case(seed, L, d, H, pt, prefix, new, n_pos=None, n_time=8, bf16=False, shuffle_pages=True,
               n_scale=None):
    """Weights, requests, shuffled page tables, timestamps and inputs for a small step."""
    rng, rng_perm, rng_in = (np.random.default_rng([seed, k]) for k in range(3))  # independent streams
    total = [p + t for p, t in zip(prefix, new)]
    n_pos = n_pos or max(total)
    cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale or float(max(total)), 1e-6, bf16)
    w = synth.make_weights(rng, L, d, H, n_pos, n_time, bf16)
    reqs, n_pt, n_ts, n_rows = synth.make_requests(prefix, new, pt)
    n_pages = n_pt + 3
    perm = rng_perm.permutation(n_pages) if shuffle_pages else np.arange(n_pages)
    page_tables = perm[:n_pt].astype(np.int32)
    ts = np.concatenate([synth.timestamps(rng_in, s) for s in total]) if total else np.zeros(0, np.int64)
    x = rng_in.standard_normal((n_rows, d)).astype(np.float32)
    if bf16:
        x = synth.as_bf16_values(x)
    kv = np.zeros(n_pages * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    return cfg, w, reqs, page_tables, ts, x, kv


def torch_layer_dense(cfg, w, l, X, Kc, Vc, ts, P, store):
    """One HSTU layer for one request in dense-matrix form with torch fp64 library ops.
    X [T][d] new tokens; Kc, Vc [P][d] cached prefix (may be empty). Returns Y, K_all, V_all."""
    d, H = cfg.d, cfg.H
    dh = d // H
    T = X.shape[0]
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    Xn = F.layer_norm(X, (d,), t64(w["ln1_g"][l]), t64(w["ln1_b"][l]), cfg.eps)
    Z = F.silu(Xn @ t64(w["w1"][l]) + t64(w["b1"][l]))
    U, V, Q, K = Z[:, :d], Z[:, d:2 * d], Z[:, 2 * d:3 * d], Z[:, 3 * d:]
    K, V = store(K), store(V)
    Ka, Va = torch.cat([Kc, K]), torch.cat([Vc, V])
    S = P + T
    tt = torch.from_numpy(np.asarray(ts, dtype=np.int64))
    qpos = torch.arange(P, S)[:, None]
    kpos = torch.arange(S)[None, :]
    rel = (qpos - kpos).clamp(min=0, max=cfg.n_pos - 1)
    dt = (tt[P:S][:, None] - tt[None, :S]).clamp(min=1)
    bucket = torch.tensor([[int(v).bit_length() - 1 for v in row] for row in dt.tolist()]).clamp(max=cfg.n_time - 1)
    mask = (kpos <= qpos).to(torch.float64)
    O = torch.zeros(T, d, dtype=torch.float64)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        sc = Q[:, sl] @ Ka[:, sl].T + t64(w["pos"][l, h])[rel] + t64(w["time"][l, h])[bucket]
        A = F.silu(sc) * mask / cfg.n_scale
        O[:, sl] = A @ Va[:, sl]
    G = F.layer_norm(O, (d,), t64(w["ln2_g"][l]), t64(w["ln2_b"][l]), cfg.eps) * U
    Y = X + G @ t64(w["w2"][l]) + t64(w["b2"][l])
    return Y, Ka, Va


def torch_step_dense(cfg, w, prefix, new, x, ts_all, reqs, store):
    outs = []
    for (P, T, pto, tso, xo) in reqs:
        assert P == 0
        X = torch.from_numpy(x[xo:xo + T].astype(np.float64))
        for l in range(cfg.L):
            X, _, _ = torch_layer_dense(cfg, w, l, X, torch.zeros(0, cfg.d, dtype=torch.float64),
                                        torch.zeros(0, cfg.d, dtype=torch.float64), ts_all[tso:tso + T], 0, store)
        outs.append(X.numpy())
    return np.concatenate(outs)


# --------------------------------------------------------------------------- scalar pieces
def test_bf16_rounding_matches_torch_conversion():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 20000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, -1.001953125, 3.0e38, 1e-40], dtype=np.float32),
    ]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.round_bf16(vals)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_bf16(np.float32([1.00390625]))[0] == 1.0
    assert oracle.round_bf16(np.float32([1.01171875]))[0] == 1.015625


def test_silu_matches_torch_and_its_limits():
    xs = np.linspace(-30, 30, 241)
    want = F.silu(torch.from_numpy(xs)).numpy()
    got = np.array([oracle.silu(v) for v in xs])
    assert np.allclose(got, want, rtol=1e-14, atol=1e-300)
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12 and abs(oracle.silu(-40.0)) < 1e-12


def test_time_bucket_is_integer_log2_clamped():
    for dt in list(range(0, 70)) + [2**k + o for k in range(6, 40) for o in (-1, 0, 1)]:
        want = min(max(dt, 1).bit_length() - 1, 31)
        assert oracle.time_bucket(dt, 32) == want
    assert oracle.time_bucket(-5, 32) == 0
    assert oracle.time_bucket(10**12, 8) == 7


def test_layernorm_matches_torch():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(96) * 3 + 1
    g = rng.standard_normal(96).astype(np.float32)
    b = rng.standard_normal(96).astype(np.float32)
    want = F.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(g.astype(np.float64)),
                        torch.from_numpy(b.astype(np.float64)), 1e-6).numpy()
    assert np.allclose(oracle.layernorm(x, g, b, 1e-6), want, rtol=1e-12, atol=1e-12)


def test_kv_bytes_per_token_reproduce_the_papers_range():
    g = golden()
    for lay, tok, mb in ((g["kv_layers_low"], g["kv_tokens_low"], g["kv_mb_low"]),
                         (g["kv_layers_high"], g["kv_tokens_high"], g["kv_mb_high"])):
        cfg = oracle.make_cfg(int(lay), int(g["kv_dim"]), 8, 64, 16, 8, 1.0)
        per_token = oracle.kv_elems_per_page(cfg) * g["kv_elem_bytes"] / 64
        assert per_token == 2 * lay * g["kv_dim"] * g["kv_elem_bytes"]
        assert abs(per_token * tok / 1e6 - mb) < 0.03 * mb  # 61.4 MB and 184.3 MB


def test_page_layout_offsets_are_a_bijection():
    cfg = oracle.make_cfg(3, 12, 2, 4, 16, 8, 1.0)
    dh = 6
    seen = set()
    for page in range(2):
        for l in range(3):
            for kv in range(2):
                for h in range(2):
                    for t in range(4):
                        seen.add(oracle.kv_offset(cfg, page, l, kv, h, t))
    assert len(seen) == 2 * 3 * 2 * 2 * 4
    assert min(seen) == 0 and max(seen) == 2 * oracle.kv_elems_per_page(cfg) - dh
    assert all(o % dh == 0 for o in seen)
    assert oracle.kv_offset(cfg, 1, 0, 0, 0, 0) == oracle.kv_elems_per_page(cfg)
    # [layer][K|V][head][token][d_h]: token stride d_h, head stride pt*d_h
    assert oracle.kv_offset(cfg, 0, 0, 0, 0, 1) == dh and oracle.kv_offset(cfg, 0, 0, 0, 1, 0) == 4 * dh
    assert oracle.kv_offset(cfg, 0, 0, 1, 0, 0) == 2 * 4 * dh and oracle.kv_offset(cfg, 0, 1, 0, 0, 0) == 4 * 4 * dh


# --------------------------------------------------------------------------- attention alone
def attention_brute(cfg, pos, time, P, T, pages, ts, kv, q):
    """Triple loop in Python with its own page arithmetic."""
    d, H, pt = cfg.d, cfg.H, cfg.page_tokens
    dh = d // H
    per_page = pt * 2 * cfg.L * d
    o = np.zeros((T, d))
    for h in range(H):
        for i in range(T):
            p = P + i
            for j in range(p + 1):
                base = pages[j // pt] * per_page
                koff = base + ((0 * 2 + 0) * H + h) * pt * dh + (j % pt) * dh
                voff = base + ((0 * 2 + 1) * H + h) * pt * dh + (j % pt) * dh
                s = float(np.dot(q[i, h * dh:(h + 1) * dh], kv[koff:koff + dh].astype(np.float64)))
                s += float(pos[h, min(p - j, cfg.n_pos - 1)])
                dt = max(int(ts[p] - ts[j]), 1)
                s += float(time[h, min(dt.bit_length() - 1, cfg.n_time - 1)])
                a = s / (1.0 + np.exp(-s)) / cfg.n_scale
                o[i, h * dh:(h + 1) * dh] += a * kv[voff:voff + dh].astype(np.float64)
    return o


def test_attention_against_python_triple_loop():
    rng = np.random.default_rng(2)
    cfg = oracle.make_cfg(1, 8, 2, 4, 6, 5, 13.0)
    P, T = 5, 8
    pages = np.array([3, 0, 2, 1], dtype=np.int32)
    kv = rng.standard_normal(5 * oracle.kv_elems_per_page(cfg)).astype(np.float32)
    q = rng.standard_normal((T, 8))
    pos = rng.standard_normal((2, 6)).astype(np.float32)
    time = rng.standard_normal((2, 5)).astype(np.float32)
    ts = synth.timestamps(rng, P + T)
    got = oracle.attn_paged(cfg, 0, pos, time, P, T, pages, ts, kv, q)
    want = attention_brute(cfg, pos, time, P, T, pages, ts, kv, q)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)


def test_attention_zero_query_zero_bias_gives_exact_zero():
    rng = np.random.default_rng(3)
    cfg = oracle.make_cfg(1, 8, 2, 4, 16, 8, 16.0)
    kv = rng.standard_normal(4 * oracle.kv_elems_per_page(cfg)).astype(np.float32)
    o = oracle.attn_paged(cfg, 0, np.zeros((2, 16), np.float32), np.zeros((2, 8), np.float32), 4, 9,
                          np.arange(4, dtype=np.int32), synth.timestamps(rng, 13), kv, np.zeros((9, 8)))
    assert not o.any()  # SiLU(0) = 0


def test_attention_large_scores_reduce_to_a_masked_matmul():
    # for s >> 0, SiLU(s) -> s, so O -> (1/n) * tril(Q K^T + bias) V
    rng = np.random.default_rng(4)
    d, H, pt, S = 8, 1, 4, 12
    cfg = oracle.make_cfg(1, d, H, pt, S, 4, 7.0)
    kv = np.zeros(3 * oracle.kv_elems_per_page(cfg), dtype=np.float32)
    Kmat = (rng.random((S, d)) + 2.0).astype(np.float32)
    Vmat = rng.standard_normal((S, d)).astype(np.float32)
    for j in range(S):
        kv[oracle.kv_offset(cfg, j // pt, 0, 0, 0, j % pt):][:d] = Kmat[j]
        kv[oracle.kv_offset(cfg, j // pt, 0, 1, 0, j % pt):][:d] = Vmat[j]
    q = rng.random((S, d)) + 2.0  # every score >= 8*4 + 40
    pos = np.full((1, S), 40.0, np.float32)
    o = oracle.attn_paged(cfg, 0, pos, np.zeros((1, 4), np.float32), 0, S, np.arange(3, dtype=np.int32),
                          np.arange(S, dtype=np.int64), kv, q)
    want = np.tril(q @ Kmat.astype(np.float64).T + 40.0) @ Vmat.astype(np.float64) / 7.0
    assert np.allclose(o, want, rtol=1e-12)


def test_doubling_n_halves_attention_exactly():
    rng = np.random.default_rng(5)
    args = lambda n: oracle.make_cfg(1, 8, 2, 4, 16, 8, n)
    kv = rng.standard_normal(4 * oracle.kv_elems_per_page(args(1.0))).astype(np.float32)
    q = rng.standard_normal((10, 8))
    pos = rng.standard_normal((2, 16)).astype(np.float32)
    tm = rng.standard_normal((2, 8)).astype(np.float32)
    ts = synth.timestamps(rng, 14)
    o1 = oracle.attn_paged(args(64.0), 0, pos, tm, 4, 10, np.arange(4, dtype=np.int32), ts, kv, q)
    o2 = oracle.attn_paged(args(128.0), 0, pos, tm, 4, 10, np.arange(4, dtype=np.int32), ts, kv, q)
    assert np.array_equal(o1, 2.0 * o2)


# --------------------------------------------------------------------------- whole step
@pytest.mark.parametrize("bf16", [False, True])
def test_step_matches_dense_torch_formulation(bf16):
    prefix, new = [0, 0, 0], [13, 5, 22]
    cfg, w, reqs, pts, ts, x, kv = build_case(7, 2, 16, 2, 4, prefix, new, n_pos=10, n_time=6, bf16=bf16)
    rc, out = oracle.hstu_step(cfg, w, reqs, pts, kv, x, ts)
    assert rc == oracle.OK
    if bf16:
        store = lambda a: a.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    else:
        store = lambda a: a.to(torch.float32).to(torch.float64)
    want = torch_step_dense(cfg, w, prefix, new, x, ts, reqs, store)
    assert np.allclose(out, want, rtol=1e-10, atol=1e-12)


def test_stored_kv_are_the_projections_in_the_documented_layout():
    cfg, w, reqs, pts, ts, x, kv = build_case(8, 2, 16, 2, 4, [0], [11], bf16=True)
    rc, out = oracle.hstu_step(cfg, w, reqs, pts, kv, x, ts)
    store = lambda a: a.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    X = torch.from_numpy(x.astype(np.float64))
    for l in range(2):
        Y, Ka, Va = torch_layer_dense(cfg, w, l, X, torch.zeros(0, 16, dtype=torch.float64),
                                      torch.zeros(0, 16, dtype=torch.float64), ts, 0, store)
        for j in range(11):
            for h in range(2):
                ko = oracle.kv_offset(cfg, int(pts[j // 4]), l, 0, h, j % 4)
                vo = oracle.kv_offset(cfg, int(pts[j // 4]), l, 1, h, j % 4)
                assert np.allclose(kv[ko:ko + 8], Ka[j, h * 8:(h + 1) * 8].numpy(), rtol=1e-2, atol=1e-6)
                assert np.allclose(kv[vo:vo + 8], Va[j, h * 8:(h + 1) * 8].numpy(), rtol=1e-2, atol=1e-6)
                # stored values are bf16-representable
                assert np.array_equal(kv[ko:ko + 8], synth.as_bf16_values(kv[ko:ko + 8]))
        X = Y


@pytest.mark.parametrize("bf16", [False, True])
def test_prefix_cache_equivalence_is_bit_exact(bf16):
    # step(P cached, T new) == last T rows of step(0 cached, P+T new)
    L, d, H, pt = 2, 16, 2, 4
    P, T = 9, 6
    cfg, w, reqs, pts, ts, x, kv = build_case(9, L, d, H, pt, [0], [P + T], bf16=bf16)
    rc, full = oracle.hstu_step(cfg, w, reqs, pts, kv, x, ts)
    # serve the same user in two steps on a fresh pool
    kv2 = np.zeros_like(kv)
    rc, first = oracle.hstu_step(cfg, w, [(0, P, 0, 0, 0)], pts, kv2, x[:P], ts)
    assert np.array_equal(first, full[:P])
    rc, second = oracle.hstu_step(cfg, w, [(P, T, 0, 0, 0)], pts, kv2, x[P:], ts)
    assert np.array_equal(second, full[P:])
    assert np.array_equal(kv2, kv)


def test_future_tokens_do_not_influence_earlier_rows():
    cfg, w, reqs, pts, ts, x, kv = build_case(10, 2, 16, 2, 4, [0], [14])
    rc, a = oracle.hstu_step(cfg, w, reqs, pts, kv, x, ts)
    x2 = x.copy()
    x2[9:] += 3.0
    ts2 = ts.copy()
    ts2[9:] += 100000
    rc, b = oracle.hstu_step(cfg, w, reqs, pts, np.zeros_like(kv), x2, ts2)
    assert np.array_equal(a[:9], b[:9]) and not np.array_equal(a[9:], b[9:])


def test_page_table_permutation_and_page_size_do_not_change_outputs():
    prefix, new = [0, 0], [19, 8]
    outs = []
    for pt, shuffle in ((4, False), (4, True), (16, True), (64, True)):
        cfg, w, reqs, pts, ts, x, kv = build_case(11, 2, 16, 2, pt, prefix, new, n_pos=19, shuffle_pages=shuffle,
                                                  n_scale=19.0)
        outs.append(oracle.hstu_step(cfg, w, reqs, pts, kv, x, ts)[1])
    for o in outs[1:]:
        assert np.array_equal(outs[0], o)


def test_requests_are_independent_and_threads_do_not_change_results():
    prefix, new = [0, 0, 0, 0], [7, 12, 3, 9]
    cfg, w, reqs, pts, ts, x, kv = build_case(12, 2, 16, 2, 4, prefix, new, n_pos=12, n_scale=12.0)
    kv1, kv4, kva = kv.copy(), kv.copy(), kv.copy()
    rc, one = oracle.hstu_step(cfg, w, reqs, pts, kv1, x, ts, threads=1)
    rc, many = oracle.hstu_step(cfg, w, reqs, pts, kv4, x, ts, threads=4)
    assert np.array_equal(one, many) and np.array_equal(kv1, kv4)
    # requests served alone, one call each (the threads then work inside the request: over its tokens in
    # the projections, over (head, query) pairs in the attention), give the same rows and the same stored K,V
    for (P, T, pto, tso, xo) in reqs:
        rc, alone = oracle.hstu_step(cfg, w, [(P, T, pto, tso, 0)], pts, kva, x[xo:xo + T], ts, threads=4)
        assert np.array_equal(alone, one[xo:xo + T])
    assert np.array_equal(kva, kv1)


def test_page_table_out_of_range_is_rejected():
    cfg, w, reqs, pts, ts, x, kv = build_case(13, 1, 16, 2, 4, [0], [6])
    bad = pts.copy()
    bad[1] = 10**6
    assert oracle.hstu_step(cfg, w, reqs, bad, kv, x, ts)[0] == oracle.ERANGE
