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
    for (b, g), op in res.items():
        if not np.array_equal(sel[b, g], op.sel):
            assert harness.boundary_gap(op, cfg.k) < 1e-6, (cfg, b, g)
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
        s = oracle.decision_scores(oracle.score(q1[b, g * cfg.G:(g + 1) * cfg.G], op.dig))
        t = table0[b, g].copy()
        wrb, wrs, web, n = oracle.recall_plan(s, cfg.k, t[:len(s)])
        ok = (nr[b, g] == n and np.array_equal(rb[b, g], wrb) and np.array_equal(rs[b, g], wrs)
              and np.array_equal(eb[b, g], web) and np.array_equal(got_t[b, g], t))
        if not ok:
            r = oracle.rank(s)
            gaps = [abs(s[r[j]] - s[r[j + 1]]) / max(abs(s[r[j]]), 1e-300) for j in range(len(s) - 1)]
            assert gaps and min(gaps) < 1e-6, (cfg, b, g)
