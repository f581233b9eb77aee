"""The host-side worker (Alg. 1 CPUAttn) against the oracle's partial attention (CPU only).

Partials are compared through what is unique: the normalised o and lse = m + ln l.  Tolerance: the
worker accumulates in binary32 over at most a few thousand tokens, 1e-5 relative to the value scale.
"""
import numpy as np
import pytest

import oracle
from paper_2603_27138_amd import host as H
from paper_2603_27138_amd import workload as W


def _case(dtype, B, Hq, Hkv, d, S, mb, k, seed, ctx=None):
    rng = np.random.default_rng(seed)
    st = lambda x: W.to_storage(x.astype(np.float32), dtype)
    ctx = np.asarray(ctx if ctx is not None else rng.integers(1, mb * S + 1, size=B), dtype=np.int32)
    q = st(rng.standard_normal((B, Hq, d)))
    kb = st(rng.standard_normal((B, Hkv, mb, S, d)))
    vb = st(rng.standard_normal((B, Hkv, mb, S, d)))
    sel = np.full((B, Hkv, k), -1, dtype=np.int32)
    n = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        nb = (int(ctx[b]) + S - 1) // S
        for g in range(Hkv):
            cnt = int(rng.integers(0, min(k, nb) + 1))
            sel[b, g, :cnt] = np.sort(rng.permutation(nb)[:cnt])
            n[b, g] = cnt
    return ctx, q, kb, vb, sel, n


def _run(worker, dtype, B, Hq, Hkv, d, S, mb, k, ctx, q, kb, vb, sel, n):
    p = H.HostProblem(B, Hq, Hkv, d, S, H.F32 if dtype == "f32" else H.BF16, mb, k, 0.0)
    o = np.full((B, Hq, d), np.nan, dtype=np.float32)
    m = np.full((B, Hq), np.nan, dtype=np.float32)
    l = np.full((B, Hq), np.nan, dtype=np.float32)
    worker.submit(p, q, kb, vb, sel, n, ctx, o, m, l)
    sec = worker.wait()
    assert sec >= 0.0 and worker.done()
    return o, m, l


def _check(dtype, B, Hq, Hkv, d, S, mb, k, ctx, q, kb, vb, sel, n, o, m, l, tol=2e-5):
    G = Hq // Hkv
    sm = 1.0 / np.sqrt(d)
    for b in range(B):
        for g in range(Hkv):
            K = kb[b, g].reshape(mb * S, d)
            V = vb[b, g].reshape(mb * S, d)
            for h in range(G):
                hq = g * G + h
                wo, wm, wl = oracle.partial_attn(q[b, hq], K, V, sel[b, g], int(ctx[b]), S, sm)
                if wl == 0.0:
                    assert l[b, hq] == 0.0 and m[b, hq] == -np.inf and (o[b, hq] == 0).all()
                    continue
                assert np.abs(o[b, hq] - wo).max() <= tol * max(1.0, np.abs(wo).max()), (b, g, h)
                lse, wlse = m[b, hq] + np.log(l[b, hq]), wm + np.log(wl)
                assert abs(lse - wlse) <= tol * max(1.0, abs(wlse)), (b, g, h)


@pytest.fixture(scope="module")
def worker():
    w = H.HostWorker(4)
    yield w
    w.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,Hq,Hkv,d,S,mb,k", [(3, 8, 2, 128, 32, 9, 5), (2, 4, 4, 64, 16, 7, 7), (1, 16, 1, 128, 64, 3, 2),
                                              (5, 6, 3, 8, 1, 12, 4)])
def test_host_partial_matches_oracle(worker, dtype, B, Hq, Hkv, d, S, mb, k):
    case = _case(dtype, B, Hq, Hkv, d, S, mb, k, seed=B * 100 + d)
    out = _run(worker, dtype, B, Hq, Hkv, d, S, mb, k, *case)
    _check(dtype, B, Hq, Hkv, d, S, mb, k, *case, *out)


def test_host_partial_masks_the_tail_and_skips_bad_entries(worker):
    B, Hq, Hkv, d, S, mb, k = 1, 2, 1, 8, 4, 4, 4
    ctx, q, kb, vb, sel, n = _case("f32", B, Hq, Hkv, d, S, mb, k, seed=3, ctx=[10])   # block 2 has 2 valid tokens
    sel[0, 0] = [0, 2, 3, 9]     # block 3 lies beyond the context, 9 is no block
    n[0, 0] = 4
    o, m, l = _run(worker, "f32", B, Hq, Hkv, d, S, mb, k, ctx, q, kb, vb, sel, n)
    good = np.array([0, 2, -1, -1], dtype=np.int32)
    for h in range(Hq):
        wo, wm, wl = oracle.partial_attn(q[0, h], kb[0, 0].reshape(-1, d), vb[0, 0].reshape(-1, d), good, 10, S,
                                         1.0 / np.sqrt(d))
        assert np.abs(o[0, h] - wo).max() < 1e-5 and abs(m[0, h] + np.log(l[0, h]) - wm - np.log(wl)) < 1e-5


def test_host_worker_many_jobs_back_to_back_and_busy_refusal():
    # more pairs than threads, jobs of different shapes one after the other on the same pool
    w = H.HostWorker(3)
    try:
        for it, (B, Hkv) in enumerate([(8, 4), (1, 1), (6, 2), (2, 8)] * 3):
            shape = (B, 2 * Hkv, Hkv, 64, 16, 6, 3)
            case = _case("bf16", *shape, seed=it)
            out = _run(w, "bf16", *shape, *case)
            _check("bf16", *shape, *case, *out)
        # one job may wait behind the running one (see the test of two outstanding jobs below); a further
        # one is refused
        shape = (64, 8, 8, 128, 32, 40, 40)
        ctx, q, kb, vb, sel, n = _case("bf16", *shape, seed=99, ctx=[40 * 32] * 64)
        p = H.HostProblem(*shape[:5], H.BF16, shape[5], shape[6], 0.0)
        o = np.zeros((64, 8, 128), np.float32); m = np.zeros((64, 8), np.float32); l = np.zeros((64, 8), np.float32)
        o2, m2, l2 = o.copy(), m.copy(), l.copy()
        w.submit(p, q, kb, vb, sel, n, ctx, o, m, l)
        w.submit(p, q, kb, vb, sel, n, ctx, o2, m2, l2)
        if not w.done():
            o3, m3, l3 = o.copy(), m.copy(), l.copy()
            try:
                w.submit(p, q, kb, vb, sel, n, ctx, o3, m3, l3)
                w.wait()                       # the first job had ended meanwhile: three to wait for
            except RuntimeError as e:
                assert "-6" in str(e)
        w.wait()
        w.wait()
        assert w.done() and np.array_equal(o, o2) and np.array_equal(l, l2)
    finally:
        w.close()


def test_host_worker_rejects_bad_arguments():
    w = H.HostWorker(1)
    try:
        shape = (1, 2, 1, 8, 4, 2, 2)
        case = _case("f32", *shape, seed=1)
        for bad in (dict(d=12), dict(S=65), dict(Hq=3, Hkv=2), dict(dtype=7)):
            f = dict(B=1, Hq=2, Hkv=1, d=8, S=4, dtype=0, max_blocks=2, k=2, sm_scale=0.0)
            f.update(bad)
            p = H.HostProblem(*f.values())
            o = np.zeros((1, 2, 8), np.float32); m = np.zeros((1, 2), np.float32); l = np.zeros((1, 2), np.float32)
            with pytest.raises(RuntimeError):
                w.submit(p, case[1], case[2], case[3], case[4], case[5], case[0], o, m, l)
    finally:
        w.close()
    with pytest.raises(RuntimeError):
        H.HostWorker(0)


# ---------------------------------------------------------------- recall staging (Sec. 3.4)

def _plan(rng, pairs, mb, k, counts):
    blk = np.full((pairs, k), -1, dtype=np.int32)
    n = np.asarray(counts, dtype=np.int32)
    for p in range(pairs):
        m = max(0, min(int(n[p]), k))
        blk[p, :m] = rng.permutation(mb)[:m]
    return blk, n


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("threads", [1, 5])
def test_stage_recall_equals_the_oracle_packing(dtype, threads):
    rng = np.random.default_rng(61)
    B, Hkv, mb, S, d, k = 3, 2, 11, 16, 64, 7
    st = lambda x: W.to_storage(x.astype(np.float32), dtype)
    kb, vb = st(rng.standard_normal((B, Hkv, mb, S, d))), st(rng.standard_normal((B, Hkv, mb, S, d)))
    blk, n = _plan(rng, B * Hkv, mb, k, [3, 0, 7, 1, 12, -2])      # 12 is clamped to k, -2 to 0
    blk[2, 4] = mb                                                   # no such block: its tile stays as it was
    want, want_off = oracle.recall_stage(kb.reshape(B * Hkv, mb, S, d), vb.reshape(B * Hkv, mb, S, d), blk, n)
    p = H.HostProblem(B, 4, Hkv, d, S, H.F32 if dtype == "f32" else H.BF16, mb, k, 0.0)
    staged = np.zeros_like(want)
    off = np.full(B * Hkv, -7, dtype=np.int32)
    w = H.HostWorker(threads)
    try:
        total = w.stage_recall(p, kb, vb, blk.reshape(B, Hkv, k), n.reshape(B, Hkv), staged, off)
        w.wait()
    finally:
        w.close()
    assert total == len(want) == 3 + 0 + 7 + 1 + 7 + 0
    assert np.array_equal(off, want_off) and np.array_equal(staged, want)


def test_stage_recall_rejects_a_short_buffer_and_takes_an_empty_plan():
    B, Hkv, mb, S, d, k = 1, 2, 4, 2, 8, 3
    kb = np.zeros((B, Hkv, mb, S, d), dtype=np.float32)
    blk = np.zeros((B, Hkv, k), dtype=np.int32)
    p = H.HostProblem(B, 2, Hkv, d, S, H.F32, mb, k, 0.0)
    off = np.zeros(B * Hkv, dtype=np.int32)
    w = H.HostWorker(2)
    try:
        short = np.zeros((2, 2, S, d), dtype=np.float32)             # room for 2 tiles, the plan has 3
        with pytest.raises(RuntimeError):
            w.stage_recall(p, kb, kb, blk, np.array([[2, 1]], dtype=np.int32), short, off)
        assert w.done()
        assert w.stage_recall(p, kb, kb, blk, np.zeros((B, Hkv), dtype=np.int32), short, off) == 0
        assert w.done() and off.tolist() == [0, 0]
        # the pool still takes an attention job afterwards
        assert w.stage_recall(p, kb, kb, blk, np.array([[1, 1]], dtype=np.int32), short, off) == 2
        w.wait()
        assert off.tolist() == [0, 1]
    finally:
        w.close()


def test_two_jobs_outstanding_are_run_in_order_and_a_third_is_refused():
    """Alg. 1 spawns layer i+1's host job while layer i's may still be running: the worker takes one job
    behind the running one, wait() reports them oldest first, and both give what they give alone."""
    dims = dict(dtype="bf16", B=3, Hq=8, Hkv=2, d=128, S=32, mb=48, k=20)
    cases = [_case(seed=s, **dims) for s in (21, 22, 23)]
    worker = H.HostWorker(3)
    try:
        alone = [_run(worker, **dims, **dict(zip(("ctx", "q", "kb", "vb", "sel", "n"), c))) for c in cases]
        p = H.HostProblem(dims["B"], dims["Hq"], dims["Hkv"], dims["d"], dims["S"], H.BF16, dims["mb"], dims["k"], 0.0)
        outs = []
        for rounds in range(20):                      # many times: the hand-over between jobs is a race if it is wrong
            outs = []
            for c in cases[:2]:
                ctx, q, kb, vb, sel, n = c
                o = np.full((dims["B"], dims["Hq"], dims["d"]), np.nan, dtype=np.float32)
                m = np.full((dims["B"], dims["Hq"]), np.nan, dtype=np.float32)
                l = np.full((dims["B"], dims["Hq"]), np.nan, dtype=np.float32)
                worker.submit(p, q, kb, vb, sel, n, ctx, o, m, l)
                outs.append((o, m, l))
            # a third job while one may be running and one waits: refused, unless the first is done already
            ctx, q, kb, vb, sel, n = cases[2]
            o3 = np.zeros((dims["B"], dims["Hq"], dims["d"]), dtype=np.float32)
            m3, l3 = np.zeros((dims["B"], dims["Hq"]), dtype=np.float32), np.zeros((dims["B"], dims["Hq"]), dtype=np.float32)
            try:
                worker.submit(p, q, kb, vb, sel, n, ctx, o3, m3, l3)
                third = True
            except RuntimeError as e:
                assert "-6" in str(e)
                third = False
            assert worker.wait() >= 0.0 and worker.wait() >= 0.0
            if third:
                worker.wait()
            assert worker.done()
            for (o, m, l), (wo, wm, wl) in zip(outs, alone[:2]):
                assert np.array_equal(o, wo) and np.array_equal(m, wm) and np.array_equal(l, wl)
            if third:
                assert np.array_equal(o3, alone[2][0])
        assert worker.wait() == 0.0                   # nothing outstanding: returns at once
    finally:
        worker.close()
