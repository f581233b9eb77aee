"""Device-side test plumbing: upload a workload, allocate outputs, call the binding.

No arithmetic of the method; the expected values come from tests/harness.py (oracle).
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2603_27138_amd import binding as B
from paper_2603_27138_amd import workload as W


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy storage array -> CUDA tensor (uint16 bit patterns become bfloat16)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class Dev:
    """One layer's inputs and outputs in device memory."""

    def __init__(self, wl: W.Workload, k_blocks: bool = True):
        cfg = wl.cfg
        self.cfg, self.wl = cfg, wl
        self.tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        self.ctx_len = torch.from_numpy(wl.ctx_len).cuda()
        self.p = B.make_problem(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, B.F32 if cfg.dtype == "f32" else B.BF16,
                                cfg.max_blocks, cfg.k, self.ctx_len, 0.0)
        self.ws = B.alloc_workspace(self.p)
        self.q = to_dev(wl.q)
        self.block_table = torch.from_numpy(wl.block_table).cuda()
        self.n_slots = wl.n_slots
        self.k_pool = to_dev(wl.k_pool)
        self.v_pool = to_dev(wl.v_pool)
        pairs = (cfg.B, cfg.Hkv)
        self.digest = torch.zeros(*pairs, cfg.max_blocks, 2, cfg.d, dtype=self.tdt, device="cuda")
        if k_blocks:
            kb = np.full((cfg.B, cfg.Hkv, cfg.max_blocks, cfg.S, cfg.d), W._GARBAGE[cfg.dtype],
                         dtype=wl.k_pool.dtype)
            for (b, g) in wl.K:
                kb[b, g, :cfg.nb(b)] = wl.blocks_padded(b, g, "K")
            self.k_blocks = to_dev(kb)
        self.scores = torch.full((*pairs, cfg.max_blocks), float("nan"), dtype=torch.float32, device="cuda")
        i32 = dict(dtype=torch.int32, device="cuda")
        self.sel_all = torch.full((*pairs, cfg.k), -7, **i32)
        self.sel_gpu = torch.full((*pairs, cfg.k), -7, **i32)
        self.slot_gpu = torch.full((*pairs, cfg.k), -7, **i32)
        self.sel_host = torch.full((*pairs, cfg.k), -7, **i32)
        self.n_gpu = torch.full(pairs, -7, **i32)
        self.n_host = torch.full(pairs, -7, **i32)
        f32 = dict(dtype=torch.float32, device="cuda")
        self.o = torch.full((cfg.B, cfg.Hq, cfg.d), float("nan"), **f32)
        self.m = torch.full((cfg.B, cfg.Hq), float("nan"), **f32)
        self.l = torch.full((cfg.B, cfg.Hq), float("nan"), **f32)
        self.host_o = torch.zeros((cfg.B, cfg.Hq, cfg.d), **f32)
        self.host_m = torch.full((cfg.B, cfg.Hq), float("-inf"), **f32)
        self.host_l = torch.zeros((cfg.B, cfg.Hq), **f32)
        self.out = torch.zeros((cfg.B, cfg.Hq, cfg.d), dtype=self.tdt, device="cuda")
        self.lse = torch.full((cfg.B, cfg.Hq), float("nan"), **f32)
        self.recall_blk = torch.full((*pairs, cfg.k), -7, **i32)
        self.recall_slot = torch.full((*pairs, cfg.k), -7, **i32)
        self.evict_blk = torch.full((*pairs, cfg.k), -7, **i32)
        self.n_recall = torch.full(pairs, -7, **i32)

    # ---- the calls, one per boundary entry point
    def build_digests(self):
        B.build_digests(self.p, self.k_blocks, self.digest)

    def score(self, q=None):
        B.score_blocks(self.p, self.q if q is None else q, self.digest, self.scores, self.ws)

    def select(self, scores=None):
        B.select_topk(self.p, self.scores if scores is None else scores, self.block_table, self.sel_all,
                      self.sel_gpu, self.slot_gpu, self.n_gpu, self.sel_host, self.n_host, self.ws)

    def attn(self, q=None):
        B.sparse_decode_attn(self.p, self.q if q is None else q, self.k_pool, self.v_pool, self.n_slots,
                             self.sel_gpu, self.slot_gpu, self.n_gpu, self.o, self.m, self.l, self.ws)

    def merge(self, host=True):
        if host:
            B.merge_partials(self.p, self.o, self.m, self.l, self.host_o, self.host_m, self.host_l, self.out,
                             self.lse)
        else:
            B.merge_partials(self.p, self.o, self.m, self.l, None, None, None, self.out, self.lse)

    def layer_step(self, q=None, host=True):
        h = (self.host_o, self.host_m, self.host_l) if host else (None, None, None)
        B.layer_step(self.p, self.q if q is None else q, self.digest, self.block_table, self.k_pool, self.v_pool,
                     self.n_slots, *h, self.scores, self.sel_all, self.sel_gpu, self.slot_gpu, self.n_gpu,
                     self.sel_host, self.n_host, self.out, self.lse, self.ws)

    def recall(self, q=None):
        B.periodic_recall(self.p, self.q if q is None else q, self.digest, self.block_table, self.recall_blk,
                          self.recall_slot, self.evict_blk, self.n_recall, self.ws)

    # ---- uploads of oracle-made inputs
    def set_digest_from_oracle(self, res):
        cfg = self.cfg
        dg = np.zeros((cfg.B, cfg.Hkv, cfg.max_blocks, 2, cfg.d), dtype=self.wl.k_pool.dtype)
        for (b, g), op in res.items():
            dg[b, g, :op.dig.shape[0]] = op.dig
        self.digest.copy_(to_dev(dg))

    def set_selection_from_oracle(self, res, table=None):
        cfg = self.cfg
        table = self.wl.block_table if table is None else table
        sg = np.full((cfg.B, cfg.Hkv, cfg.k), -1, dtype=np.int32)
        sl = np.full((cfg.B, cfg.Hkv, cfg.k), -1, dtype=np.int32)
        ng = np.zeros((cfg.B, cfg.Hkv), dtype=np.int32)
        for (b, g), op in res.items():
            sg[b, g] = op.sel_gpu
            ng[b, g] = op.n_gpu
            sl[b, g, :op.n_gpu] = table[b, g, op.sel_gpu[:op.n_gpu]]
        self.sel_gpu.copy_(torch.from_numpy(sg))
        self.slot_gpu.copy_(torch.from_numpy(sl))
        self.n_gpu.copy_(torch.from_numpy(ng))

    def set_host_partials_from_oracle(self, res):
        cfg = self.cfg
        ho = np.zeros((cfg.B, cfg.Hq, cfg.d), dtype=np.float32)
        hm = np.full((cfg.B, cfg.Hq), -np.inf, dtype=np.float32)
        hl = np.zeros((cfg.B, cfg.Hq), dtype=np.float32)
        for (b, g), op in res.items():
            for h in range(cfg.G):
                o, m, l = op.host_part[h]
                ho[b, g * cfg.G + h], hm[b, g * cfg.G + h], hl[b, g * cfg.G + h] = o, m, l
        self.host_o.copy_(torch.from_numpy(ho))
        self.host_m.copy_(torch.from_numpy(hm))
        self.host_l.copy_(torch.from_numpy(hl))
