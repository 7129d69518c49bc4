"""GPU parity of hstu_step / hstu_attn_paged against the fp64 oracle.

Tolerances: tests/parity.py (two relative measures per output row, 1e-4 for fp32 models; for bf16
models, whose intermediates are rounded to bf16 while the oracle rounds only the stored K,V, 2e-2 in
the row's max norm)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_04450_amd import binding as B
from paper_2605_04450_amd import device as Hn
from paper_2605_04450_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

class Case:
    """One model + pool on the device and the matching oracle state."""

    def __init__(self, seed, L, d, H, pt, bf16, n_pos, n_time, n_scale, n_pages):
        self.L, self.d, self.H, self.pt, self.bf16 = L, d, H, pt, bf16
        self.rng = np.random.default_rng(seed)
        self.elem = B.ELEM_BF16 if bf16 else B.ELEM_F32
        self.w = synth.make_weights(self.rng, L, d, H, n_pos, n_time, bf16)
        self.model = Hn.Model(L, d, H, self.elem, pt, n_pos, n_time, n_scale, self.w)
        self.cfg = oracle.make_cfg(L, d, H, pt, n_pos, n_time, n_scale, 1e-6, bf16)
        esz = 2 if bf16 else 4
        self.n_pages = n_pages
        self.pool = Hn.Pool(n_pages, self.model.page_size(), d * esz, self.elem, pt, 32, None, 0.25, zero_fill=False)
        self.kv = np.zeros(n_pages * oracle.kv_elems_per_page(self.cfg), dtype=np.float32)
        self.mem = self.pool.mem.view(torch.bfloat16 if bf16 else torch.float32)

    def inputs(self, prefix, new, shuffle=True):
        reqs, n_pt, n_ts, N = synth.make_requests(prefix, new, self.pt)
        first_kv = self.n_pages // 4  # pages below are EMB
        perm_rng = np.random.default_rng(12345)  # its own stream: placement must not change the data drawn below
        perm = first_kv + (perm_rng.permutation(self.n_pages - first_kv) if shuffle else np.arange(self.n_pages - first_kv))
        assert n_pt <= len(perm)
        pts = perm[:n_pt].astype(np.int32)
        ts = np.concatenate([synth.timestamps(self.rng, p + t) for p, t in zip(prefix, new)])
        x = self.rng.standard_normal((N, self.d)).astype(np.float32)
        if self.bf16:
            x = synth.as_bf16_values(x)
        return reqs, pts, ts, x

    def run_gpu(self, reqs, pts, ts, x):
        xd = torch.from_numpy(x).to(Hn.DEV).to(Hn.torch_dtype(self.elem))
        out = torch.empty_like(xd)
        rc = B.hstu_step(self.pool.h, self.model.h, reqs, torch.from_numpy(pts).to(Hn.DEV), xd,
                         torch.from_numpy(ts).to(Hn.DEV), out)
        assert rc == B.OK, (rc, B.last_error())
        torch.cuda.synchronize()
        return out.float().cpu().numpy()

    def run_oracle(self, reqs, pts, ts, x):
        rc, ref = oracle.hstu_step(self.cfg, self.w, reqs, pts, self.kv, x, ts)
        assert rc == oracle.OK
        return ref

    def oracle_kv_rows(self, pages, S, layer):
        """K, V [S][d] of one layer as the oracle stored them."""
        dh = self.d // self.H
        K = np.zeros((S, self.d), np.float32)
        V = np.zeros((S, self.d), np.float32)
        for j in range(S):
            for h in range(self.H):
                ko = oracle.kv_offset(self.cfg, int(pages[j // self.pt]), layer, 0, h, j % self.pt)
                vo = oracle.kv_offset(self.cfg, int(pages[j // self.pt]), layer, 1, h, j % self.pt)
                K[j, h * dh:(h + 1) * dh] = self.kv[ko:ko + dh]
                V[j, h * dh:(h + 1) * dh] = self.kv[vo:vo + dh]
        return K, V

    def close(self):
        self.model.close()
        self.pool.close()


def assert_close(got, ref, bf16, what=""):
    parity.assert_close(got, ref, bf16, what)


def test_tiny_config_fp32_full_output_and_stored_kv():
    # Tiny config: 1 layer, d = 64, 2 heads, fp32, KV page 16 tokens, 4 requests x 256 tokens
    c = Case(1, 1, 64, 2, 16, False, 256, 32, 256.0, 128)
    reqs, pts, ts, x = c.inputs([0, 0, 0, 0], [256, 256, 256, 256])
    got, ref = c.run_gpu(reqs, pts, ts, x), c.run_oracle(reqs, pts, ts, x)
    assert_close(got, ref, False, "tiny")
    for (P, T, pto, tso, xo) in reqs[:2]:
        pages = pts[pto:pto + 16]
        Kg, Vg = Hn.read_kv(c.mem, c.L, c.d, c.H, c.pt, pages, 256, 0)
        Ko, Vo = c.oracle_kv_rows(pages, 256, 0)
        assert np.allclose(Kg.cpu().numpy(), Ko, rtol=1e-4, atol=1e-6)
        assert np.allclose(Vg.cpu().numpy(), Vo, rtol=1e-4, atol=1e-6)
    assert c.pool.stats()["bad_pages"] == 0
    c.close()


@pytest.mark.parametrize("L,d,H,pt,lens", [
    (2, 128, 2, 16, [130, 64, 257, 1, 33]),
    (1, 256, 4, 64, [300, 129, 64]),
    (3, 64, 1, 8, [70, 5]),
])
def test_bf16_prefill_ragged_lengths(L, d, H, pt, lens):
    c = Case(2, L, d, H, pt, True, max(lens), 16, float(max(lens)), 256)
    reqs, pts, ts, x = c.inputs([0] * len(lens), lens)
    got, ref = c.run_gpu(reqs, pts, ts, x), c.run_oracle(reqs, pts, ts, x)
    assert_close(got, ref, True, "bf16 prefill")
    # stored K,V of the last layer agree with the oracle's to bf16 resolution
    (P, T, pto, tso, xo) = reqs[0]
    pages = pts[pto:pto + (T + pt - 1) // pt]
    Kg, Vg = Hn.read_kv(c.mem, c.L, c.d, c.H, c.pt, pages, T, L - 1)
    Ko, Vo = c.oracle_kv_rows(pages, T, L - 1)
    assert_close(Kg.float().cpu().numpy(), Ko, True, "bf16 prefill stored K")
    assert_close(Vg.float().cpu().numpy(), Vo, True, "bf16 prefill stored V")
    assert c.pool.stats()["bad_pages"] == 0
    c.close()


def test_bf16_long_sequences_use_split_key_ranges():
    # long enough that query tiles are cut into several key-range items whose fp32 partial
    # outputs are summed by the reduction pass; second step scores a short tail on a long prefix
    c = Case(8, 1, 128, 2, 64, True, 4096, 32, 4096.0, 256)
    reqs, pts, ts, x = c.inputs([0, 0, 0], [2500, 900, 3000 + 300])
    first = [(0, 2500, reqs[0][2], reqs[0][3], 0), (0, 900, reqs[1][2], reqs[1][3], 2500),
             (0, 3000, reqs[2][2], reqs[2][3], 3400)]
    xa = np.concatenate([x[:2500], x[2500:3400], x[3400:6400]])
    ga, oa = c.run_gpu(first, pts, ts, xa), c.run_oracle(first, pts, ts, xa)
    assert_close(ga, oa, True, "long prefill")
    second = [(3000, 300, reqs[2][2], reqs[2][3], 0)]
    xb = x[6400:6700]
    gb, ob = c.run_gpu(second, pts, ts, xb), c.run_oracle(second, pts, ts, xb)
    assert_close(gb, ob, True, "short tail on a long cached prefix")
    assert c.pool.stats()["bad_pages"] == 0
    c.close()


@pytest.mark.parametrize("bf16,L,d,H,pt,first,more", [
    (False, 2, 64, 2, 16, [200, 77, 130], [60, 140, 1]),
    (True, 2, 128, 2, 16, [200, 77, 130], [60, 140, 1]),
    # the width of the long-history configuration (d = 512, 8 heads): separate LayerNorm + GEMM kernels,
    # ragged lengths, row tiles with a tail, a request that gets nothing in the second step
    (True, 2, 512, 8, 64, [300, 129, 64, 1, 515], [70, 1, 130, 64, 0]),
])
def test_prefix_reuse_two_steps(bf16, L, d, H, pt, first, more):
    # step 1 prefills, step 2 scores new tokens against the cached prefix (KV reuse)
    c = Case(3, L, d, H, pt, bf16, 1024, 16, 1024.0, 128)
    nreq = len(first)
    reqs1, pts, ts, x_all = c.inputs([0] * nreq, [a + b for a, b in zip(first, more)])
    # carve the two steps out of the same page tables / timestamps
    def step_inputs(prefix, new, take_from):
        reqs, rows = [], []
        xo = 0
        for r, (P_, T_, pto, tso, xoff) in enumerate(reqs1):
            reqs.append((prefix[r], new[r], pto, tso, xo))
            rows.append(x_all[xoff + take_from[r]: xoff + take_from[r] + new[r]])
            xo += new[r]
        return reqs, np.concatenate(rows)
    ra, xa = step_inputs([0] * nreq, first, [0] * nreq)
    rb, xb = step_inputs(first, more, first)
    ga, oa = c.run_gpu(ra, pts, ts, xa), c.run_oracle(ra, pts, ts, xa)
    gb, ob = c.run_gpu(rb, pts, ts, xb), c.run_oracle(rb, pts, ts, xb)
    assert_close(ga, oa, bf16, "d=%d step 1" % d)
    assert_close(gb, ob, bf16, "d=%d step 2 on cached prefix" % d)
    # stored K,V of the last layer (both steps' tokens) agree with the oracle's to the storage type's resolution
    (P_, T_, pto, tso, xo) = reqs1[0]
    S = first[0] + more[0]
    pages = pts[pto:pto + (S + pt - 1) // pt]
    Kg, Vg = Hn.read_kv(c.mem, c.L, c.d, c.H, c.pt, pages, S, L - 1)
    Ko, Vo = c.oracle_kv_rows(pages, S, L - 1)
    assert_close(Kg.float().cpu().numpy(), Ko, bf16, "d=%d stored K" % d)
    assert_close(Vg.float().cpu().numpy(), Vo, bf16, "d=%d stored V" % d)
    assert c.pool.stats()["bad_pages"] == 0
    c.close()


@pytest.mark.parametrize("bf16,d,H,pt", [(True, 128, 2, 16), (True, 64, 1, 64), (False, 64, 2, 16), (False, 48, 3, 4)])
def test_attention_alone_on_synthetic_cache(bf16, d, H, pt):
    P, T = [300, 0, 65], [140, 129, 1]
    c = Case(4, 1, d, H, pt, bf16, 256, 12, 300.0, 256)  # n_pos < sequence length: the clamp is used
    reqs, pts, ts, x = c.inputs(P, T)
    dh = d // H
    rng = c.rng
    q = rng.standard_normal((sum(T), d)).astype(np.float32)
    if bf16:
        q = synth.as_bf16_values(q)
    dt = Hn.torch_dtype(c.elem)
    for (P_, T_, pto, tso, xo) in reqs:
        S = P_ + T_
        pages = pts[pto:pto + (S + pt - 1) // pt]
        k = (rng.standard_normal((S, d)) / np.sqrt(np.sqrt(dh))).astype(np.float32)
        v = rng.standard_normal((S, d)).astype(np.float32)
        if bf16:
            k, v = synth.as_bf16_values(k), synth.as_bf16_values(v)
        Hn.write_prefix_kv(c.mem, 1, d, H, pt, pages, torch.from_numpy(k).to(Hn.DEV).to(dt),
                           torch.from_numpy(v).to(Hn.DEV).to(dt), 0)
        for j in range(S):
            for h in range(H):
                ko = oracle.kv_offset(c.cfg, int(pages[j // pt]), 0, 0, h, j % pt)
                vo = oracle.kv_offset(c.cfg, int(pages[j // pt]), 0, 1, h, j % pt)
                c.kv[ko:ko + dh] = k[j, h * dh:(h + 1) * dh]
                c.kv[vo:vo + dh] = v[j, h * dh:(h + 1) * dh]
    qd = torch.from_numpy(q).to(Hn.DEV).to(dt)
    o = torch.empty_like(qd)
    rc = B.hstu_attn_paged(c.pool.h, c.model.h, 0, reqs, torch.from_numpy(pts).to(Hn.DEV), qd,
                           torch.from_numpy(ts).to(Hn.DEV), o)
    assert rc == B.OK, B.last_error()
    torch.cuda.synchronize()
    got = o.float().cpu().numpy()
    for (P_, T_, pto, tso, xo) in reqs:
        S = P_ + T_
        ref = oracle.attn_paged(c.cfg, 0, c.w["pos"][0], c.w["time"][0], P_, T_, pts[pto:pto + (S + pt - 1) // pt],
                                ts[tso:tso + S], c.kv, q[xo:xo + T_].astype(np.float64))
        assert_close(got[xo:xo + T_], ref, bf16, "attention")
    c.close()


def test_outputs_do_not_depend_on_page_placement_or_page_size():
    outs = []
    for pt, shuffle in ((16, False), (16, True), (64, True)):
        c = Case(5, 2, 128, 2, pt, True, 300, 16, 300.0, 128)
        reqs, pts, ts, x = c.inputs([0, 0], [300, 100], shuffle=shuffle)
        outs.append(c.run_gpu(reqs, pts, ts, x))
        c.close()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


@pytest.mark.parametrize("bf16,d", [(False, 64), (True, 128), (True, 64)])
def test_bad_page_ids_are_skipped_and_counted(bf16, d):
    # fp32 kernels, the fused bf16 layer halves (d = 128) and the separate bf16 LayerNorm + GEMM kernels (d = 64)
    c = Case(6, 1, d, d // 64 if bf16 else 2, 16, bf16, 64, 8, 64.0, 64)
    reqs, pts, ts, x = c.inputs([0], [40])
    bad = pts.copy()
    bad[1] = 10**6
    out = c.run_gpu(reqs, bad, ts, x)
    assert np.isfinite(out).all()
    assert c.pool.stats()["bad_pages"] > 0
    c.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_requests_with_decreasing_timestamps_follow_the_oracle(bf16):
    # the interface asks for non-decreasing timestamps; a request that breaks this is still served like the oracle
    # serves it (a negative gap falls into bucket 0), by the general time path, and counted
    c = Case(15, 1, 128 if bf16 else 64, 2, 16, bf16, 512, 16, 512.0, 128)
    prefix, new = [0, 100, 0], [200, 90, 140]
    reqs, pts, ts, x = c.inputs(prefix, new)
    ts = ts.copy()
    (P, T, pto, tso, xo) = reqs[1]
    seg = ts[tso:tso + P + T]
    ts[tso:tso + P + T] = seg[np.random.default_rng(3).permutation(P + T)]   # request 1: any order
    ts[reqs[2][3] + 70] = ts[reqs[2][3] + 69] - 5000                        # request 2: one step back
    if P:  # request 1's cached prefix: one prefill step with the same timestamps
        pre = [(0, P, pto, tso, 0)]
        xp = c.rng.standard_normal((P, c.d)).astype(np.float32)
        xp = synth.as_bf16_values(xp) if bf16 else xp
        assert_close(c.run_gpu(pre, pts, ts, xp), c.run_oracle(pre, pts, ts, xp), bf16, "unordered timestamps, prefill")
    got, ref = c.run_gpu(reqs, pts, ts, x), c.run_oracle(reqs, pts, ts, x)
    assert_close(got, ref, bf16, "unordered timestamps")
    assert c.pool.stats()["unordered_ts"] == 3  # request 1 twice (prefill and step), request 2 once
    c.close()


def test_shape_errors_are_reported():
    c = Case(7, 1, 64, 2, 16, False, 64, 8, 64.0, 64)
    reqs, pts, ts, x = c.inputs([0], [40])
    xd = torch.from_numpy(x).to(Hn.DEV)
    out = torch.empty_like(xd)
    ptd, tsd = torch.from_numpy(pts).to(Hn.DEV), torch.from_numpy(ts).to(Hn.DEV)
    assert B.hstu_step(c.pool.h, c.model.h, [(0, 40, 0, 0, 5)], ptd, xd, tsd, out) == B.EINVAL   # rows not packed
    assert B.hstu_step(c.pool.h, c.model.h, [(0, 400, 0, 0, 0)], ptd, xd, tsd, out) == B.EINVAL  # table too short
    w = synth.make_weights(c.rng, 1, 64, 2, 64, 8, False)
    other = Hn.Model(1, 64, 2, B.ELEM_F32, 32, 64, 8, 64.0, w)  # different page size
    assert B.hstu_step(c.pool.h, other.h, reqs, ptd, xd, tsd, out) == B.EINVAL
    rc, h = B.hstu_model_create(1, 96, 2, B.ELEM_BF16, 16, 64, 8, 64.0, 1e-6, other.w)  # d_h = 48 in bf16
    assert rc == B.EINVAL
    other.close()
    c.close()


MIXED = [3000, 1700, 4096, 2500, 64, 3900, 2048, 3333, 2900, 4000, 1500, 3800, 1]  # 34 837 tokens


@pytest.mark.parametrize("L,d,H,lens", [
    (2, 128, 2, MIXED),             # fused layer halves
    (1, 512, 8, MIXED),             # separate LayerNorm + GEMM kernels
    (1, 128, 2, [30000, 5, 3000]),  # one request holds nearly all the work: the cuts fall right behind it
    (1, 128, 2, [20000, 15000]),    # fewer requests than pipelines: stays one pipeline
    (1, 128, 2, [33000, 0, 0, 7]),  # requests without new tokens
])
def test_pipelined_step_equals_the_single_pipeline_step_bit_for_bit(L, d, H, lens):
    # A batch of 32 768 or more new tokens runs as three pipelines on three streams, unless kernels are being timed.
    # Same work items, same chunking, same summation order: the outputs and the stored K,V must be identical,
    # also when further work is queued on the caller's stream right behind the step.  (Parity of the pipelined
    # step with the oracle: the full-size Mid test in test_gpu_configs.py.)
    c = Case(31, L, d, H, 64, True, 4096, 16, 4096.0, 1024)
    reqs, pts, ts, x = c.inputs([0] * len(lens), lens)
    xd = torch.from_numpy(x).to(Hn.DEV).to(torch.bfloat16)
    ptd, tsd = torch.from_numpy(pts).to(Hn.DEV), torch.from_numpy(ts).to(Hn.DEV)
    outs, kvs = [], []
    for timed in (0, 1, 0):
        c.pool.mem.zero_()
        B.racer_prof_enable(c.pool.h, timed)
        out = torch.empty_like(xd)
        assert B.hstu_step(c.pool.h, c.model.h, reqs, ptd, xd, tsd, out) == B.OK, B.last_error()
        follow = out.float().sum(dim=1)  # queued behind the step on the same stream: must see the finished output
        torch.cuda.synchronize()
        assert torch.equal(follow, out.float().sum(dim=1))
        outs.append(out.clone())
        kvs.append(c.pool.mem.clone())
    B.racer_prof_enable(c.pool.h, 0)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
    assert torch.equal(outs[0].view(torch.int16), outs[2].view(torch.int16))
    assert torch.equal(kvs[0], kvs[1]) and torch.equal(kvs[0], kvs[2])
    c.close()


def test_pipelined_step_random_batches_match_the_single_pipeline():
    # random request counts and lengths (total 33k-60k new tokens, so the pipelines are used), one pool reused
    # from batch to batch without waiting in between
    c = Case(77, 1, 128, 2, 64, True, 2048, 16, 2048.0, 2048)
    rng = np.random.default_rng(5)
    piped, serial = [], []
    batches = []
    for b in range(10):
        n_req = int(rng.integers(3, 40))
        lens = rng.integers(1, 3000, size=n_req)
        lens = (lens * (rng.integers(33000, 60000) / lens.sum())).astype(np.int64) + 1
        reqs, pts, ts, x = c.inputs([0] * n_req, lens.tolist())
        batches.append((reqs, torch.from_numpy(pts).to(Hn.DEV), torch.from_numpy(ts).to(Hn.DEV),
                        torch.from_numpy(x).to(Hn.DEV).to(torch.bfloat16)))
    for timed, outs in ((0, piped), (1, serial)):
        B.racer_prof_enable(c.pool.h, timed)
        for reqs, ptd, tsd, xd in batches:  # back to back: the next step's lists and kernels queue behind this one
            out = torch.empty_like(xd)
            assert B.hstu_step(c.pool.h, c.model.h, reqs, ptd, xd, tsd, out) == B.OK, B.last_error()
            outs.append(out)
        torch.cuda.synchronize()
    B.racer_prof_enable(c.pool.h, 0)
    for k, (a, b_) in enumerate(zip(piped, serial)):
        assert torch.equal(a.view(torch.int16), b_.view(torch.int16)), k
    c.close()
