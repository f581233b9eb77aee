"""Seeded random shapes through the whole step and the recall plan: combinations of batch, group size,
head dimension, block size, element type, ragged lengths (zero included), budget and residency that the
named configurations do not list.  Same bars as everywhere: selections and plans exact (a mismatch only
below a 1e-6 relative boundary gap), outputs within the attention tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_27138_amd import workload as W
from tests import harness
from tests.gpu_harness import Dev, to_dev, to_np

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}


def random_config(i):
    rng = np.random.default_rng([20260327, i])
    dtype = ["bf16", "f32"][int(rng.integers(2))]
    d = [64, 128][int(rng.integers(2))]
    S = [16, 32, 64][int(rng.integers(3))]
    G = [1, 2, 4, 8, 16][int(rng.integers(5))]
    Hkv = int(rng.integers(1, 4))
    Bn = int(rng.integers(1, 4))
    max_tok = int(rng.integers(1, 40)) * S
    ctx = tuple(int(rng.integers(0, max_tok + 1)) if rng.random() < 0.8 else max_tok for _ in range(Bn))
    if max(ctx) == 0:
        ctx = ctx[:-1] + (S + 1,)
    k = int(rng.integers(1, 24))
    p_host = float([0.0, 0.3, 0.5, 0.8, 1.0][int(rng.integers(5))])
    return W.shrink(W.tiny(), name=f"random-{i}", B=Bn, Hq=G * Hkv, Hkv=Hkv, d=d, S=S, dtype=dtype, ctx=ctx, k=k,
                    p_host=p_host, planted=0.1, seed=777 + i)


@pytest.mark.parametrize("i", range(32))
def test_random_shape(i):
    cfg = random_config(i)
    wl = W.generate(cfg)
    res = harness.run_all(wl)
    dev = Dev(wl, k_blocks=True)
    dev.build_digests()
    dev.set_host_partials_from_oracle(res)
    dev.layer_step()
    sel = dev.sel_all.cpu().numpy()
    ng, nh = dev.n_gpu.cpu().numpy(), dev.n_host.cpu().numpy()
    out = W.storage_to_f32(to_np(dev.out)).astype(np.float64)
    lse = dev.lse.cpu().numpy()
    excused = 0
    for (b, g), op in res.items():
        if not np.array_equal(sel[b, g], op.sel):
            assert harness.boundary_gap(op, cfg.k) < 1e-6, (cfg, b, g)
            excused += 1
            continue
        assert ng[b, g] == op.n_gpu and nh[b, g] == op.n_host, (cfg, b, g)
        for h in range(cfg.G):
            want, wlse = op.out[h]
            hq = g * cfg.G + h
            assert np.abs(out[b, hq] - want).max() <= TOL[cfg.dtype], (cfg, b, g, h)
            if np.isneginf(wlse):
                assert np.isneginf(lse[b, hq])
            else:
                assert abs(lse[b, hq] - wlse) <= 2e-3 * max(1.0, abs(wlse)), (cfg, b, g, h)
    # the recall plan for a drifted query
    q1 = W.gen_q(cfg, 0, step=3)
    table0 = wl.block_table.copy()
    dev.recall(to_dev(q1))
    got_t = dev.block_table.cpu().numpy()
    rb, rs, eb, nr = (t.cpu().numpy() for t in (dev.recall_blk, dev.recall_slot, dev.evict_blk, dev.n_recall))
    for (b, g), op in res.items():
        s64 = oracle.score(q1[b, g * cfg.G:(g + 1) * cfg.G], op.dig)
        s = oracle.decision_scores(s64)
        t = table0[b, g].copy()
        wrb, wrs, web, n = oracle.recall_plan(s, cfg.k, t[:len(s)])
        ok = (nr[b, g] == n and np.array_equal(rb[b, g], wrb) and np.array_equal(rs[b, g], wrs)
              and np.array_equal(eb[b, g], web) and np.array_equal(got_t[b, g], t))
        if not ok:      # only a gap that decides the plan may excuse
            assert harness.plan_gap(s64, s, cfg.k, table0[b, g]) < 1e-6, (cfg, b, g)
            excused += 1
    assert harness.few(excused, 2 * len(res)), excused


def _unit_oracle(wl, b, heads, g, sums, variant):
    """One selection unit (the heads that share a selection) with the variant's scoring: returns
    (decision scores after always-kept blocks, selection, per-head (out, lse), per-head host partial)."""
    cfg = wl.cfg
    K, V, ctx = wl.K[(b, g)], wl.V[(b, g)], int(cfg.ctx[b])
    qu = wl.q[b, heads[0]:heads[-1] + 1]
    if variant["digest_kind"]:
        s = oracle.score_mean(qu, sums[(b, g)], ctx, cfg.S)
    elif variant["group_max"]:
        s = oracle.score_max(qu, oracle.digest(K, ctx, cfg.S))
    else:
        s = oracle.score(qu, oracle.digest(K, ctx, cfg.S))
    f = oracle.force_blocks(oracle.decision_scores(s), variant["n_sink"], variant["n_tail"])
    s = np.where(np.isfinite(f), s, f)      # exact scores, always-kept blocks at +inf like the decision's
    sel = oracle.select(f, cfg.k)
    sg, ng, sh, nh = oracle.split(sel, wl.block_table[b, g])
    outs, hosts = [], []
    for hq in heads:
        pg = oracle.partial_attn(wl.q[b, hq], K, V, sg, ctx, cfg.S, cfg.sm_scale)
        ph = oracle.partial_attn(wl.q[b, hq], K, V, sh, ctx, cfg.S, cfg.sm_scale)
        ph32 = (ph[0].astype(np.float32).astype(np.float64), float(np.float32(ph[1])), float(np.float32(ph[2])))
        hosts.append(ph32)
        outs.append(oracle.merge(pg[0], pg[1], pg[2], *ph32))
    return (f, s), sel, outs, hosts


@pytest.mark.parametrize("i", range(24))
def test_random_shape_with_random_variant(i):
    """The selection variants in random combination on random shapes: always-kept blocks, maximum over
    the group's heads, a selection per query head, mean-pooled digests (the last not with the maximum)."""
    from paper_2603_27138_amd import binding as B
    cfg = random_config(100 + i)
    rng = np.random.default_rng([4242, i])
    variant = dict(n_sink=int(rng.integers(0, 3)), n_tail=int(rng.integers(0, 3)), per_head=int(rng.integers(2)),
                   digest_kind=int(rng.integers(2)), group_max=0)
    if not variant["digest_kind"]:
        variant["group_max"] = int(rng.integers(2))
    print(f"[random variant] {cfg.name} {cfg.dtype} d{cfg.d} S{cfg.S} B{cfg.B} Hq{cfg.Hq} Hkv{cfg.Hkv} ctx{cfg.ctx} k{cfg.k} {variant}",
          flush=True)
    wl = W.generate(cfg)
    dev = Dev(wl, k_blocks=True)
    code = B.F32 if cfg.dtype == "f32" else B.BF16
    p = B.make_problem(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, code, cfg.max_blocks, cfg.k, dev.ctx_len, 0.0, **variant)
    ws = B.alloc_workspace(p)
    sums = {}
    if variant["digest_kind"]:
        digest = torch.zeros(cfg.B, cfg.Hkv, cfg.max_blocks, cfg.d, dtype=torch.float32, device="cuda")
        sums = {(b, g): oracle.digest_sum(wl.K[(b, g)], int(cfg.ctx[b]), cfg.S) for (b, g) in wl.K}
    else:
        digest = dev.digest
    B.build_digests(p, dev.k_blocks, digest)
    rows = cfg.Hq if variant["per_head"] else cfg.Hkv
    units = {}
    for b in range(cfg.B):
        for r in range(rows):
            heads = [r] if variant["per_head"] else list(range(r * cfg.G, (r + 1) * cfg.G))
            units[(b, r)] = (heads, _unit_oracle(wl, b, heads, heads[0] // cfg.G, sums, variant))
    ho = np.zeros((cfg.B, cfg.Hq, cfg.d), dtype=np.float32)
    hm = np.full((cfg.B, cfg.Hq), -np.inf, dtype=np.float32)
    hl = np.zeros((cfg.B, cfg.Hq), dtype=np.float32)
    for (b, r), (heads, (_, _, _, hosts)) in units.items():
        for hq, hp in zip(heads, hosts):
            ho[b, hq], hm[b, hq], hl[b, hq] = hp
    host = [torch.from_numpy(a).cuda() for a in (ho, hm, hl)]
    i32 = dict(dtype=torch.int32, device="cuda")
    scores = torch.full((cfg.B, rows, cfg.max_blocks), float("nan"), dtype=torch.float32, device="cuda")
    sel_all, sel_gpu, slot_gpu, sel_host = (torch.full((cfg.B, rows, cfg.k), -7, **i32) for _ in range(4))
    n_gpu, n_host = torch.full((cfg.B, rows), -7, **i32), torch.full((cfg.B, rows), -7, **i32)
    B.layer_step(p, dev.q, digest, dev.block_table, dev.k_pool, dev.v_pool, dev.n_slots, *host, scores, sel_all, sel_gpu,
                 slot_gpu, n_gpu, sel_host, n_host, dev.out, dev.lse, ws)
    torch.cuda.synchronize()
    sel = sel_all.cpu().numpy()
    out = W.storage_to_f32(to_np(dev.out)).astype(np.float64)
    lse = dev.lse.cpu().numpy()
    excused = 0
    for (b, r), (heads, ((f, s64), wsel, outs, _)) in units.items():
        if not np.array_equal(sel[b, r], wsel):
            # only the gap between the last kept and the first dropped block may excuse
            assert harness.selection_gap(s64, f, cfg.k) < 1e-6, (cfg, variant, b, r)
            excused += 1
            continue
        for hq, (want, wlse) in zip(heads, outs):
            assert np.abs(out[b, hq] - want).max() <= TOL[cfg.dtype], (cfg, variant, b, hq)
            if np.isneginf(wlse):
                assert np.isneginf(lse[b, hq])
            else:
                assert abs(lse[b, hq] - wlse) <= 2e-3 * max(1.0, abs(wlse)), (cfg, variant, b, hq)
    assert harness.few(excused, len(units)), excused
