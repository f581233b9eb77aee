"""Mean-pooled digests (stored as binary32 sums of a block's keys) on the device against the oracle:
the build and the append bit for bit, the scores within one binary32 rounding, and the whole
layer-step (selection exact up to the near-tie rule, outputs within the attention tolerance).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_27138_amd import binding as B
from paper_2603_27138_amd import workload as W
from tests import harness
from tests.gpu_harness import Dev, to_dev, to_np

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def _configs():
    return [
        W.tiny(),
        W.shrink(W.qwen3_32b(B=2, ctx=4096), name="mean-c3"),
        W.shrink(W.qwen3_32b(B=3, ctx=0), name="mean-ragged", ctx=(1000, 37, 2111), k=24, p_host=0.3),
        W.shrink(W.tiny(), name="mean-f32-ragged", B=2, Hq=8, Hkv=2, ctx=(517, 2040), k=20, p_host=0.25),
        W.shrink(W.qwen3_8b(B=2, ctx=2048), name="mean-d64-s16", d=64, S=16, k=32),
        W.shrink(W.qwen3_8b(B=1, ctx=8192), name="mean-s64", S=64, Hq=16, k=16),
        W.shrink(W.qwen3_8b(B=3, ctx=0), name="mean-empty-sequence", ctx=(0, 64, 1), k=4, p_host=0.5),
    ]


CFGS = _configs()


def _problem(cfg, dev, **kw):
    code = B.F32 if cfg.dtype == "f32" else B.BF16
    return B.make_problem(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, code, cfg.max_blocks, cfg.k, dev.ctx_len, 0.0,
                          digest_kind=1, **kw)


def _oracle_sums(wl):
    cfg = wl.cfg
    sums = np.zeros((cfg.B, cfg.Hkv, cfg.max_blocks, cfg.d), dtype=np.float32)
    for (b, g) in wl.K:
        s = oracle.digest_sum(wl.K[(b, g)], int(cfg.ctx[b]), cfg.S)
        sums[b, g, :len(s)] = s
    return sums


@pytest.mark.parametrize("cfg", CFGS, ids=[c.name for c in CFGS])
def test_mean_digest_build_score_and_step(cfg):
    print(f"[mean digest] {cfg.name}", flush=True)
    wl = W.generate(cfg)
    dev = Dev(wl)
    p = _problem(cfg, dev)
    want_sums = _oracle_sums(wl)
    # build: bit for bit (rows of blocks beyond a context are left as they were)
    dsum = torch.full((cfg.B, cfg.Hkv, cfg.max_blocks, cfg.d), 7.0, dtype=torch.float32, device="cuda")
    B.build_digests(p, dev.k_blocks, dsum)
    got = dsum.cpu().numpy()
    for b in range(cfg.B):
        nb = cfg.nb(b)
        assert np.array_equal(got[b, :, :nb].view(np.uint32), want_sums[b, :, :nb].view(np.uint32)), b
        assert (got[b, :, nb:] == 7.0).all()
    # scores
    ws = B.alloc_workspace(p)
    B.score_blocks(p, dev.q, dsum, dev.scores, ws)
    got_s = dev.scores.cpu().numpy()
    res = {}
    for (b, g) in wl.K:
        ctx, nb = int(cfg.ctx[b]), cfg.nb(b)
        qg = wl.q[b, g * cfg.G:(g + 1) * cfg.G]
        s = oracle.score_mean(qg, want_sums[b, g, :nb], ctx, cfg.S)
        s32 = oracle.decision_scores(s)
        if nb:
            # one binary32 rounding of the binary64 value (sums of products may cancel: a floor relative to
            # the pair's largest score covers the binary64 rounding of the two summation orders)
            err = np.abs(got_s[b, g, :nb].astype(np.float64) - s)
            assert (err <= 1e-7 * np.abs(s) + 1e-10 * np.abs(s).max()).all(), (b, g)
        assert np.isneginf(got_s[b, g, nb:]).all()
        sel = oracle.select(s32, cfg.k)
        sg, ng, sh, nh = oracle.split(sel, wl.block_table[b, g])
        outs, hosts = [], []
        for h in range(cfg.G):
            pg = oracle.partial_attn(qg[h], wl.K[(b, g)], wl.V[(b, g)], sg, ctx, cfg.S, cfg.sm_scale)
            ph = oracle.partial_attn(qg[h], wl.K[(b, g)], wl.V[(b, g)], sh, ctx, cfg.S, cfg.sm_scale)
            ph32 = (ph[0].astype(np.float32).astype(np.float64), float(np.float32(ph[1])), float(np.float32(ph[2])))
            hosts.append(ph32)
            outs.append(oracle.merge(pg[0], pg[1], pg[2], *ph32)[0])
        res[(b, g)] = (s, s32, sel, outs, hosts)
    # the fused step with the host partials of the oracle's selection
    ho = np.zeros((cfg.B, cfg.Hq, cfg.d), dtype=np.float32)
    hm = np.full((cfg.B, cfg.Hq), -np.inf, dtype=np.float32)
    hl = np.zeros((cfg.B, cfg.Hq), dtype=np.float32)
    for (b, g), (_, _, _, _, hosts) in res.items():
        for h in range(cfg.G):
            ho[b, g * cfg.G + h], hm[b, g * cfg.G + h], hl[b, g * cfg.G + h] = hosts[h]
    host = [torch.from_numpy(a).cuda() for a in (ho, hm, hl)]
    B.layer_step(p, dev.q, dsum, dev.block_table, dev.k_pool, dev.v_pool, dev.n_slots, *host, dev.scores, dev.sel_all,
                 dev.sel_gpu, dev.slot_gpu, dev.n_gpu, dev.sel_host, dev.n_host, dev.out, dev.lse, ws)
    torch.cuda.synchronize()
    sel_dev = dev.sel_all.cpu().numpy()
    out = W.storage_to_f32(to_np(dev.out)).astype(np.float64)
    differ_from_minmax = False
    for (b, g), (s, s32, sel, outs, _) in res.items():
        if not np.array_equal(sel_dev[b, g], sel):
            nb, r = len(s), oracle.rank(s32)
            gap = abs(s[r[cfg.k - 1]] - s[r[cfg.k]]) / max(abs(s[r[cfg.k - 1]]), abs(s[r[cfg.k]]), 1e-300) if cfg.k < nb else 1.0
            assert gap < 1e-6, (b, g)
            continue
        for h in range(cfg.G):
            assert np.abs(out[b, g * cfg.G + h] - outs[h]).max() <= TOL[cfg.dtype], (b, g, h)
        differ_from_minmax |= not np.array_equal(sel, harness.run_pair(wl, b, g, attention=False).sel)
    if all(cfg.nb(b) > cfg.k for b in range(cfg.B)):
        assert differ_from_minmax      # otherwise these inputs could not tell the two digests apart
    # the mean digest has no maximum-over-heads variant
    with pytest.raises(B.ScoutError):
        B.score_blocks(_problem(cfg, dev, group_max=1), dev.q, dsum, dev.scores, ws)


@pytest.mark.parametrize("dtype,d,S", [("bf16", 128, 32), ("f32", 64, 16)])
def test_mean_digest_append_equals_rebuild(dtype, d, S):
    rng = np.random.default_rng(5)
    Bn, Hkv, mb = 3, 2, 4
    ctx = np.array([0, S - 1, 2 * S + 3], dtype=np.int32)
    steps = S + 5
    st = lambda x: W.to_storage(x.astype(np.float32), dtype)
    code = B.F32 if dtype == "f32" else B.BF16
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    keys = {(b, g): st(rng.standard_normal((mb * S, d))) for b in range(Bn) for g in range(Hkv)}
    sums = np.full((Bn, Hkv, mb, d), 3.0, dtype=np.float32)
    for (b, g), K in keys.items():
        s = oracle.digest_sum(K[:ctx[b]], int(ctx[b]), S)
        sums[b, g, :len(s)] = s
    d_ctx = torch.from_numpy(ctx.copy()).cuda()
    d_sums = torch.from_numpy(sums.copy()).cuda()
    table = torch.full((Bn, Hkv, mb), -1, dtype=torch.int32, device="cuda")
    pool = torch.zeros(1, S, d, dtype=tdt, device="cuda")
    new_slot = torch.full((Bn, Hkv), -1, dtype=torch.int32, device="cuda")        # every block stays on the host
    p = B.make_problem(Bn, Hkv, Hkv, d, S, code, mb, 2, d_ctx, 0.0, digest_kind=1)
    cur = ctx.copy()
    for step in range(steps):
        k_new = np.stack([np.stack([keys[(b, g)][min(cur[b], mb * S - 1)] for g in range(Hkv)]) for b in range(Bn)])
        for b in range(Bn):
            for g in range(Hkv):
                oracle.append_sum(S, int(cur[b]), k_new[b, g], sums[b, g])
            if cur[b] < mb * S:
                cur[b] += 1
        dk = to_dev(k_new)
        B.append_token(p, d_ctx, dk, dk, new_slot, d_sums, table, pool, pool, 0)
    torch.cuda.synchronize()
    assert np.array_equal(d_ctx.cpu().numpy(), cur)
    assert np.array_equal(d_sums.cpu().numpy().view(np.uint32), sums.view(np.uint32))
    for (b, g), K in keys.items():      # and both equal the digest built at once from the finished keys
        s = oracle.digest_sum(K[:cur[b]], int(cur[b]), S)
        assert np.array_equal(sums[b, g, :len(s)].view(np.uint32), s.view(np.uint32))
