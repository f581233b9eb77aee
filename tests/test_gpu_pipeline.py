"""The layer-ahead pipeline (Sec. 3.3, Algorithm 1) against the oracle's statement of the same
algorithm: blocks selected with the predicted query, the GPU's partial with the real query over the
resident selected blocks, the host's partial with the predicted query over the offloaded ones
(handed over in binary32), merged.  Selections bit-exact, outputs within the attention tolerance.
Also reports (does not bound tightly) how far the pipelined output is from the step computed with
the real query throughout: the approximation the paper's method accepts.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_27138_amd import binding as B
from paper_2603_27138_amd import pipeline as P
from paper_2603_27138_amd import workload as W
from tests.gpu_harness import to_dev, to_np

pytestmark = pytest.mark.gpu


def _pinned(a: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
    return t.pin_memory()


def _layer(wl):
    cfg = wl.cfg
    shape = (cfg.B, cfg.Hkv, cfg.max_blocks, cfg.S, cfg.d)
    kb, vb = np.zeros(shape, wl.k_pool.dtype), np.zeros(shape, wl.k_pool.dtype)
    dig = np.zeros((cfg.B, cfg.Hkv, cfg.max_blocks, 2, cfg.d), wl.k_pool.dtype)
    digs = {}
    for (b, g) in wl.K:
        nb = cfg.nb(b)
        kb[b, g, :nb], vb[b, g, :nb] = wl.blocks_padded(b, g, "K"), wl.blocks_padded(b, g, "V")
        digs[(b, g)] = oracle.digest(wl.K[(b, g)], int(cfg.ctx[b]), cfg.S)
        dig[b, g, :nb] = digs[(b, g)]
    layer = P.Layer(to_dev(dig), torch.from_numpy(wl.block_table).cuda(), to_dev(wl.k_pool), to_dev(wl.v_pool),
                    wl.n_slots, _pinned(kb), _pinned(vb))
    return layer, digs


def _oracle_alg1(wl, digs, q, q_sel, q_host):
    """Per pair: (sel, per-head merged output) with the selection taken with q_sel, the resident part
    attended with q and the offloaded part with q_host."""
    cfg = wl.cfg
    res = {}
    for (b, g) in wl.K:
        sl = slice(g * cfg.G, (g + 1) * cfg.G)
        s32 = oracle.decision_scores(oracle.score(q_sel[b, sl], digs[(b, g)]))
        sel = oracle.select(s32, cfg.k)
        sg, ng, sh, nh = oracle.split(sel, wl.block_table[b, g])
        ctx = int(cfg.ctx[b])
        outs = []
        for h in range(cfg.G):
            pg = oracle.partial_attn(q[b, sl][h], wl.K[(b, g)], wl.V[(b, g)], sg, ctx, cfg.S, cfg.sm_scale)
            ph = oracle.partial_attn(q_host[b, sl][h], wl.K[(b, g)], wl.V[(b, g)], sh, ctx, cfg.S, cfg.sm_scale)
            ph32 = (ph[0].astype(np.float32).astype(np.float64), float(np.float32(ph[1])), float(np.float32(ph[2])))
            outs.append(oracle.merge(pg[0], pg[1], pg[2], *ph32)[0])
        res[(b, g)] = (sel, outs, s32)
    return res


@pytest.mark.parametrize("dtype,tol", [("bf16", 2e-2), ("f32", 2e-5)])
def test_pipeline_matches_algorithm_1(dtype, tol):
    base = W.qwen3_32b(B=2, ctx=4096) if dtype == "bf16" else W.tiny()
    cfg = W.shrink(base, k=16, p_host=0.5, name=f"pipe-{dtype}")
    n_layers = 3
    wls = [W.generate(cfg, layer=i) for i in range(n_layers)]
    built = [_layer(wl) for wl in wls]
    layers = [x[0] for x in built]
    ctx = torch.from_numpy(wls[0].ctx_len).cuda()
    code = B.F32 if dtype == "f32" else B.BF16
    pipe = P.LayerAheadPipeline(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, code, cfg.max_blocks, cfg.k, ctx, layers,
                                n_threads=4)
    try:
        for step in range(2):
            qs = [W.gen_q(cfg, layer=i, step=step) for i in range(n_layers)]
            qps = [W.gen_q_pred(q, 0.94, seed=10 * step + i) for i, q in enumerate(qs)]
            outs = pipe.step([to_dev(q) for q in qs], [to_dev(q) for q in qps])
            torch.cuda.synchronize()
            assert len(pipe.host_seconds) == n_layers
            worst, drift = 0.0, 0.0
            for i in range(n_layers):
                want = _oracle_alg1(wls[i], built[i][1], qs[i], qps[i], qps[i])
                exact = _oracle_alg1(wls[i], built[i][1], qs[i], qs[i], qs[i])
                got = W.storage_to_f32(to_np(outs[i])).astype(np.float64)
                sel = pipe.buf[i].sel_all.cpu().numpy()
                for (b, g), (wsel, wouts, s32) in want.items():
                    if not np.array_equal(sel[b, g], wsel):
                        r = oracle.rank(s32)
                        ke = min(cfg.k, len(s32))
                        gap = abs(s32[r[ke - 1]] - s32[r[ke]]) / max(abs(s32[r[ke - 1]]), 1e-300) if ke < len(s32) else 1.0
                        assert gap < 1e-6, (step, i, b, g)
                        continue
                    for h in range(cfg.G):
                        hq = g * cfg.G + h
                        worst = max(worst, float(np.abs(got[b, hq] - wouts[h]).max()))
                        drift = max(drift, float(np.abs(got[b, hq] - exact[(b, g)][1][h]).max()))
            assert worst <= tol, (step, worst)
            print(f"pipeline {dtype} step {step}: max |out - Alg.1 oracle| = {worst:.2e}; "
                  f"max deviation from the step with the real query throughout = {drift:.2e}", flush=True)
            assert drift > worst      # the predicted query does change the result; that is the method
    finally:
        pipe.close()


def test_pipeline_with_periodic_recall():
    """Algorithm 1 with the recall of Sec. 3.4 every second step: after those steps each layer's plan is
    made with the real query, the tiles travel by the staged route beside the next layers' work, and the
    following steps select and attend on the new residency.  The oracle mirrors it by updating its copy of
    the table with its own plan; tables, pool contents, selections and outputs must agree."""
    cfg = W.shrink(W.qwen3_32b(B=2, ctx=4096), k=16, p_host=0.5, name="pipe-recall")
    n_layers, R = 3, 2
    wls = [W.generate(cfg, layer=i) for i in range(n_layers)]
    built = [_layer(wl) for wl in wls]
    layers = [x[0] for x in built]
    ctx = torch.from_numpy(wls[0].ctx_len).cuda()
    pipe = P.LayerAheadPipeline(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, B.BF16, cfg.max_blocks, cfg.k, ctx, layers,
                                n_threads=4, recall_every=R)
    moved_total = 0
    try:
        for step in range(4):
            qs = [W.gen_q(cfg, layer=i, step=step) for i in range(n_layers)]
            qps = [W.gen_q_pred(q, 0.94, seed=10 * step + i) for i, q in enumerate(qs)]
            print(f"[pipeline+recall] step {step}", flush=True)
            outs = pipe.step([to_dev(q) for q in qs], [to_dev(q) for q in qps])
            torch.cuda.synchronize()
            worst = 0.0
            for i in range(n_layers):
                wl, digs = wls[i], built[i][1]
                want = _oracle_alg1(wl, digs, qs[i], qps[i], qps[i])     # on the residency before this step's recall
                got = W.storage_to_f32(to_np(outs[i])).astype(np.float64)
                sel = pipe.buf[i].sel_all.cpu().numpy()
                for (b, g), (wsel, wouts, s32) in want.items():
                    assert np.array_equal(sel[b, g], wsel), (step, i, b, g)
                    for h in range(cfg.G):
                        worst = max(worst, float(np.abs(got[b, g * cfg.G + h] - wouts[h]).max()))
                if step % R == R - 1:                                    # the oracle's recall, real query
                    planned = 0
                    for (b, g) in wl.K:
                        s = oracle.decision_scores(oracle.score(qs[i][b, g * cfg.G:(g + 1) * cfg.G], digs[(b, g)]))
                        planned += oracle.recall_plan(s, cfg.k, wl.block_table[b, g][:len(s)])[3]
                    moved_total += planned
                    assert np.array_equal(layers[i].block_table.cpu().numpy(), wl.block_table), (step, i)
                    assert int(pipe.buf[i].n_recall.sum().item()) == planned
                    # every resident block's slot holds that block's rows
                    kp, vp = to_np(layers[i].k_pool), to_np(layers[i].v_pool)
                    for (b, g) in wl.K:
                        kb, vb = wl.blocks_padded(b, g, "K"), wl.blocks_padded(b, g, "V")
                        for j in range(cfg.nb(b)):
                            slot = wl.block_table[b, g, j]
                            if slot >= 0:
                                assert np.array_equal(kp[slot], kb[j]) and np.array_equal(vp[slot], vb[j]), (step, i, b, g, j)
            assert worst <= 2e-2, (step, worst)
            if step % R == R - 1:
                assert pipe.recalled_tiles > 0
        assert moved_total > 0
    finally:
        pipe.close()
