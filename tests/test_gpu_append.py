"""Decode append on the device against the oracle (bit for bit), and a context that grows token by
token under the whole layer-step (selection exact, outputs within the attention tolerance).

The oracle side of the second test rebuilds every digest from the finished keys with the oracle's
one-piece digest routine, so it also checks the incremental update against the definition.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_27138_amd import binding as B
from paper_2603_27138_amd import workload as W
from tests.gpu_harness import to_dev, to_np

pytestmark = pytest.mark.gpu


def _rand(rng, shape, dtype):
    return W.to_storage(rng.standard_normal(shape).astype(np.float32), dtype)


class State:
    """Cache state of a few sequences, mirrored on the host (oracle) and on the device."""

    def __init__(self, dtype, Bn, Hkv, d, S, max_blocks, ctx0, seed, host_every=3):
        self.dtype, self.Bn, self.Hkv, self.d, self.S, self.mb = dtype, Bn, Hkv, d, S, max_blocks
        self.code = oracle.F32 if dtype == "f32" else oracle.BF16
        self.rng = np.random.default_rng(seed)
        self.host_every = host_every
        self.n_slots = Bn * Hkv * max_blocks
        st = np.float32 if dtype == "f32" else np.uint16
        self.ctx = np.zeros(Bn, dtype=np.int32)
        self.dig = np.zeros((Bn, Hkv, max_blocks, 2, d), dtype=st)
        self.table = np.full((Bn, Hkv, max_blocks), -1, dtype=np.int32)
        self.kp = np.zeros((self.n_slots, S, d), dtype=st)
        self.vp = np.zeros((self.n_slots, S, d), dtype=st)
        self.hk = np.zeros((Bn, Hkv, max_blocks, S, d), dtype=st)   # the host's copy of every block
        self.hv = np.zeros((Bn, Hkv, max_blocks, S, d), dtype=st)
        self.free = list(self.rng.permutation(self.n_slots))
        self.K = {(b, g): np.zeros((max_blocks * S, d), dtype=st) for b in range(Bn) for g in range(Hkv)}
        self.V = {(b, g): np.zeros((max_blocks * S, d), dtype=st) for b in range(Bn) for g in range(Hkv)}
        # grow to the starting lengths on the host only, one sequence at a time
        for b in range(Bn):
            for _ in range(int(ctx0[b])):
                k, v, ns = self.draw(only=b)
                self.host_append(k, v, ns, only=b)
        self.upload()

    def draw(self, only=None):
        k = _rand(self.rng, (self.Bn, self.Hkv, self.d), self.dtype)
        v = _rand(self.rng, (self.Bn, self.Hkv, self.d), self.dtype)
        ns = np.full((self.Bn, self.Hkv), -5, dtype=np.int32)   # ignored unless a block opens
        for b in range(self.Bn):
            t = int(self.ctx[b])
            if (only is None or b == only) and t % self.S == 0 and t < self.mb * self.S:
                for g in range(self.Hkv):
                    host = (t // self.S + g) % self.host_every == self.host_every - 1
                    ns[b, g] = -1 if host else int(self.free.pop())
        return k, v, ns

    def host_append(self, k, v, ns, only=None):
        for b in range(self.Bn):
            if only is not None and b != only:
                continue
            t = int(self.ctx[b])
            new = t
            for g in range(self.Hkv):
                new = oracle.append(self.code, self.S, t, k[b, g].copy(), v[b, g].copy(), int(ns[b, g]),
                                    self.dig[b, g], self.table[b, g], self.kp, self.vp, self.hk[b, g], self.hv[b, g])
                if new > t:
                    self.K[(b, g)][t], self.V[(b, g)][t] = k[b, g], v[b, g]
            self.ctx[b] = new

    def upload(self):
        self.d_ctx = torch.from_numpy(self.ctx.copy()).cuda()
        self.d_dig = to_dev(self.dig.copy())
        self.d_table = torch.from_numpy(self.table.copy()).cuda()
        self.d_kp, self.d_vp = to_dev(self.kp.copy()), to_dev(self.vp.copy())
        as_t = lambda a: torch.from_numpy(a.view(np.int16).copy() if a.dtype == np.uint16 else a.copy())
        self.p_hk, self.p_hv = as_t(self.hk).pin_memory(), as_t(self.hv).pin_memory()   # read and written by the GPU

    def problem(self, Hq, k):
        return B.make_problem(self.Bn, Hq, self.Hkv, self.d, self.S, B.F32 if self.dtype == "f32" else B.BF16,
                              self.mb, k, self.d_ctx, 0.0)

    def dev_append(self, p, k, v, ns):
        B.append_token(p, self.d_ctx, to_dev(k), to_dev(v), torch.from_numpy(ns).cuda(), self.d_dig, self.d_table,
                       self.d_kp, self.d_vp, self.n_slots, self.p_hk, self.p_hv)

    def assert_same(self, tag):
        assert np.array_equal(self.d_ctx.cpu().numpy(), self.ctx), tag
        assert np.array_equal(self.d_table.cpu().numpy(), self.table), tag
        assert np.array_equal(to_np(self.d_dig), self.dig), tag
        assert np.array_equal(to_np(self.d_kp), self.kp), tag
        assert np.array_equal(to_np(self.d_vp), self.vp), tag
        torch.cuda.synchronize()
        view = lambda t: t.numpy().view(np.uint16) if self.dtype == "bf16" else t.numpy()
        assert np.array_equal(view(self.p_hk), self.hk) and np.array_equal(view(self.p_hv), self.hv), tag


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,S", [(128, 16), (64, 32), (128, 64)])
def test_append_matches_oracle_bit_for_bit(dtype, d, S):
    mb = 4
    # an empty sequence, one about to open a block, one mid-block, one full, one a token short of full
    ctx0 = [0, S - 1, S + S // 2, mb * S, mb * S - 1]
    st = State(dtype, len(ctx0), 3, d, S, mb, ctx0, seed=17)
    p = st.problem(Hq=6, k=2)
    st.assert_same("start")
    for step in range(2 * S + 3):
        k, v, ns = st.draw()
        st.host_append(k, v, ns)
        st.dev_append(p, k, v, ns)
        if step % 7 == 0 or step >= 2 * S:
            st.assert_same(step)
    assert st.ctx[3] == mb * S and st.ctx[4] == mb * S and st.ctx[0] == 2 * S + 3


def test_append_rejects_bad_arguments():
    st = State("f32", 1, 1, 64, 16, 2, [3], seed=1)
    p = st.problem(Hq=1, k=1)
    k, v, ns = st.draw()
    args = [st.d_ctx, to_dev(k), to_dev(v), torch.from_numpy(ns).cuda(), st.d_dig, st.d_table, st.d_kp, st.d_vp]
    for i in range(len(args)):
        bad = list(args)
        bad[i] = None
        with pytest.raises(B.ScoutError) as e:
            B.append_token(p, *bad, st.n_slots)
        assert e.value.code == B.EINVAL
    with pytest.raises(B.ScoutError):
        B.append_token(p, *args, -1)
    with pytest.raises(B.ScoutError):
        B.append_token(p, *args, st.n_slots, st.p_hk, None)      # the host copy is both arrays or neither
    torch.cuda.synchronize()
    st.assert_same("untouched")


@pytest.mark.parametrize("dtype,TOL", [("bf16", 2e-2), ("f32", 1e-5)])
def test_layer_step_on_a_growing_context(dtype, TOL):
    Bn, Hq, Hkv, d, S, mb, kk = 2, 8, 2, 128, 16, 12, 4
    G = Hq // Hkv
    st = State(dtype, Bn, Hkv, d, S, mb, [40, 100], seed=23, host_every=2)
    p = st.problem(Hq, kk)
    ws = B.alloc_workspace(p)
    i32 = dict(dtype=torch.int32, device="cuda")
    pairs = (Bn, Hkv)
    scores = torch.empty((*pairs, mb), dtype=torch.float32, device="cuda")
    sel_all, sel_gpu, slot_gpu, sel_host = (torch.empty((*pairs, kk), **i32) for _ in range(4))
    n_gpu, n_host = torch.empty(pairs, **i32), torch.empty(pairs, **i32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    out = torch.empty((Bn, Hq, d), dtype=tdt, device="cuda")
    lse = torch.empty((Bn, Hq), dtype=torch.float32, device="cuda")
    sm = 1.0 / np.sqrt(d)
    worst = 0.0
    for step in range(2 * S + 5):
        k, v, ns = st.draw()
        st.host_append(k, v, ns)
        st.dev_append(p, k, v, ns)
        q = _rand(st.rng, (Bn, Hq, d), dtype)
        # oracle: digests from the finished keys, then Algorithm 1
        ho = np.zeros((Bn, Hq, d), dtype=np.float32)
        hm = np.full((Bn, Hq), -np.inf, dtype=np.float32)
        hl = np.zeros((Bn, Hq), dtype=np.float32)
        want = {}
        for (b, g) in st.K:
            ctx = int(st.ctx[b])
            Kp, Vp = st.K[(b, g)], st.V[(b, g)]
            dig = oracle.digest(Kp, ctx, S)
            qg = q[b, g * G:(g + 1) * G]
            s32 = oracle.decision_scores(oracle.score(qg, dig))
            sel = oracle.select(s32, kk)
            sg, ng, sh, nh = oracle.split(sel, st.table[b, g])
            outs = []
            for h in range(G):
                pg = oracle.partial_attn(qg[h], Kp, Vp, sg, ctx, S, sm)
                ph = oracle.partial_attn(qg[h], Kp, Vp, sh, ctx, S, sm)
                ph32 = (ph[0].astype(np.float32), np.float32(ph[1]), np.float32(ph[2]))
                ho[b, g * G + h], hm[b, g * G + h], hl[b, g * G + h] = ph32
                outs.append(oracle.merge(pg[0], pg[1], pg[2], ph32[0].astype(np.float64), float(ph32[1]), float(ph32[2])))
            want[(b, g)] = (sel, ng, nh, outs)
        B.layer_step(p, to_dev(q), st.d_dig, st.d_table, st.d_kp, st.d_vp, st.n_slots, torch.from_numpy(ho).cuda(),
                     torch.from_numpy(hm).cuda(), torch.from_numpy(hl).cuda(), scores, sel_all, sel_gpu, slot_gpu,
                     n_gpu, sel_host, n_host, out, lse, ws)
        got_sel, got_ng, got_nh = sel_all.cpu().numpy(), n_gpu.cpu().numpy(), n_host.cpu().numpy()
        got = W.storage_to_f32(to_np(out)).astype(np.float64)
        for (b, g), (sel, ng, nh, outs) in want.items():
            assert np.array_equal(got_sel[b, g], sel), (step, b, g)
            assert got_ng[b, g] == ng and got_nh[b, g] == nh, (step, b, g)
            for h in range(G):
                err = float(np.abs(got[b, g * G + h] - outs[h][0]).max())
                worst = max(worst, err)
                assert err <= TOL, (step, b, g, h, err)
    st.assert_same("end")
    print(f"growing context {dtype}: worst abs err {worst:.2e}")
