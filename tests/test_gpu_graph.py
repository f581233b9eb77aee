"""The library's calls can be recorded into a HIP graph (they allocate nothing, clear nothing with memset
nodes and never synchronise): a captured layer-step, replayed several times with new queries and with
eager work in between, gives the eager result bit for bit every time."""
import numpy as np
import pytest
import torch

from paper_2603_27138_amd import workload as W
from tests import harness
from tests.gpu_harness import Dev, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["bf16", "f32"])
def test_layer_step_replays_from_a_graph(name):
    cfg = W.shrink(W.qwen3_32b(B=2, ctx=4096), name="graph-bf16", k=16) if name == "bf16" else \
        W.shrink(W.tiny(), name="graph-f32", p_host=0.25)
    wl = W.generate(cfg)
    res = harness.run_all(wl)
    dev = Dev(wl, k_blocks=False)
    dev.set_digest_from_oracle(res)
    dev.set_host_partials_from_oracle(res)
    q_static = dev.q.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            dev.layer_step(q=q_static)          # warm-up on the capture stream
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            dev.layer_step(q=q_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for step in range(4):
        q = to_dev(W.gen_q(cfg, 0, step=step))
        # eager reference into a second set of outputs
        dev.layer_step(q=q)
        torch.cuda.synchronize()
        want = (to_np(dev.out).copy(), dev.sel_all.cpu().numpy().copy(), dev.lse.cpu().numpy().copy(),
                dev.scores.cpu().numpy().copy())
        # poison the outputs, do some unrelated eager work, then replay
        dev.out.zero_(); dev.sel_all.fill_(-9); dev.lse.zero_(); dev.scores.zero_()
        junk = torch.randn(1 << 16, device="cuda").sum()
        q_static.copy_(q)
        g.replay()
        torch.cuda.synchronize()
        assert float(junk) == float(junk)
        got = (to_np(dev.out), dev.sel_all.cpu().numpy(), dev.lse.cpu().numpy(), dev.scores.cpu().numpy())
        for a, b in zip(got, want):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), step


def test_prepared_calls_replay_the_eager_result():
    """binding.prepare marshals the arguments once; replaying gives what the direct call gives."""
    from paper_2603_27138_amd import binding as B
    cfg = W.shrink(W.qwen3_32b(B=2, ctx=4096), name="prepared-bf16", k=16)
    wl = W.generate(cfg)
    res = harness.run_all(wl)
    dev = Dev(wl, k_blocks=False)
    dev.set_digest_from_oracle(res)
    dev.set_host_partials_from_oracle(res)
    call = B.prepare(dev.layer_step)
    assert len(call.calls) == 1 and float(dev.lse.isnan().sum()) > 0    # nothing has run yet
    dev.layer_step()
    torch.cuda.synchronize()
    want = (to_np(dev.out).copy(), dev.sel_all.cpu().numpy().copy())
    dev.out.zero_(); dev.sel_all.fill_(-9)
    call()
    call()
    torch.cuda.synchronize()
    assert np.array_equal(to_np(dev.out), want[0]) and np.array_equal(dev.sel_all.cpu().numpy(), want[1])
