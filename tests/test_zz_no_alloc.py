"""sparse_decode_attn_static (the entry point that allocates nothing: its scratch is a buffer inside
the library's device image) against sparse_decode_attn on the same inputs, through the C ABI: two calls
in a row on one GPU, the second with a smaller input, so that what the first left in the shared
buffer is still there when the second runs.  Same kernels, same split count, no floating-point atomics:
the results are equal bit for bit, which is inside every tolerance of the parity tests.
"""
import numpy as np
import pytest
import torch

from paper_2603_27138_amd import binding as B
from paper_2603_27138_amd import workload as W
from tests import harness
from tests.gpu_harness import Dev

pytestmark = pytest.mark.gpu


def _both(cfg, mode=(0, 0, 0)):
    """(o, m, l) of the workspace entry point and of the static one, plus the oracle's partials."""
    wl = W.generate(cfg)
    res = harness.run_all(wl)
    dev = Dev(wl, k_blocks=False)
    dev.set_selection_from_oracle(res)
    B.set_attn_mode(*mode)
    try:
        dev.attn()
        want = tuple(t.clone() for t in (dev.o, dev.m, dev.l))
        for t in (dev.o, dev.m, dev.l):
            t.fill_(float("nan"))
        B.sparse_decode_attn_static(dev.p, dev.q, dev.k_pool, dev.v_pool, dev.n_slots, dev.sel_gpu, dev.slot_gpu,
                                    dev.n_gpu, dev.o, dev.m, dev.l)
        dev.check_guards()
    finally:
        B.set_attn_mode(0, 0, 0)
    return want, (dev.o, dev.m, dev.l), res, cfg


def _check(want, got, res, cfg):
    for w, g in zip(want, got):
        assert torch.equal(w.view(torch.int32), g.view(torch.int32))
    o, m, l = (t.cpu().numpy() for t in got)
    tol = 2e-2 if cfg.dtype == "bf16" else 1e-5
    for (b, g), op in res.items():
        for h in range(cfg.G):
            wo, wm, wl_ = op.gpu_part[h]
            hq = g * cfg.G + h
            if wl_ == 0:
                assert l[b, hq] == 0 and np.isneginf(m[b, hq]) and (o[b, hq] == 0).all()
            else:
                assert np.abs(o[b, hq] - wo).max() <= tol
                assert abs(m[b, hq] + np.log(l[b, hq]) - (wm + np.log(wl_))) <= 2e-3 * max(1.0, abs(wm))


def test_two_calls_in_a_row_the_second_smaller():
    big = W.shrink(W.qwen3_32b(B=2, ctx=8192), name="static-big")                      # 16 pairs, 16 splits each
    small = W.shrink(W.qwen3_32b(B=1, ctx=2048), name="static-small", Hq=16, Hkv=2, k=16)  # 2 pairs
    _check(*_both(big))
    _check(*_both(small))
    _check(*_both(big, mode=(2, 3, 8)))
    _check(*_both(small, mode=(1, 5, 0)))       # the vector-ALU family through the same buffer


def test_fp32_and_one_workgroup_per_pair():
    _check(*_both(W.shrink(W.tiny(), name="static-f32", p_host=0.25)))                 # vector-ALU family, fp32
    _check(*_both(W.shrink(W.qwen3_32b(B=2, ctx=4096), name="static-ns1"), mode=(2, 1, 8)))   # no scratch used


def test_a_problem_beyond_the_buffer_is_refused():
    cfg = W.shrink(W.tiny(), name="static-too-big", B=2, Hq=16, Hkv=1, d=128, S=16, ctx=(64, 64), k=4, p_host=0.0)
    wl = W.generate(cfg)
    dev = Dev(wl, k_blocks=False)
    dev.set_selection_from_oracle(harness.run_all(wl))
    big = B.make_problem(64, 128, 8, 128, 16, B.F32, cfg.max_blocks, cfg.k, dev.ctx_len.repeat(32), 0.0)
    before = (dev.o.clone(), dev.m.clone(), dev.l.clone())
    with pytest.raises(B.ScoutError) as ei:
        B.sparse_decode_attn_static(big, dev.q, dev.k_pool, dev.v_pool, dev.n_slots, dev.sel_gpu, dev.slot_gpu,
                                    dev.n_gpu, dev.o, dev.m, dev.l)
    assert ei.value.code == B.ESCRATCH
    torch.cuda.synchronize()
    for a, b in zip(before, (dev.o, dev.m, dev.l)):      # nothing was launched, nothing written
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
