"""Device-side test plumbing: upload a workload, allocate outputs, call the binding.

No arithmetic of the method; the expected values come from tests/harness.py (oracle).
"""
from __future__ import annotations

import weakref

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


GUARD = 256          # bytes of pattern in front of and behind every output tensor
PATTERN = 0xA5


class Arena:
    """Output tensors carved out of one byte buffer with guard bands between them: 256 bytes of a fixed
    pattern before the first tensor, and from the last byte of every tensor to the start of the next
    one (at least 256 bytes).  A kernel that writes past either end of an output changes a guard byte,
    which check() finds with one small gather, whatever the write held."""

    def __init__(self, specs):
        """specs: (name, shape, torch dtype, fill value) per tensor, in the order they are laid out."""
        esize = {torch.float32: 4, torch.int32: 4, torch.bfloat16: 2, torch.uint8: 1}
        at, spans = GUARD, []
        for name, shape, dt, fill in specs:
            nbytes = int(np.prod(shape, dtype=np.int64)) * esize[dt]
            spans.append((name, shape, dt, fill, at, nbytes))
            at = (at + nbytes + GUARD + 255) & ~255      # the next tensor starts 256-byte aligned
        self.buf = torch.full((at,), PATTERN, dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0
        self.tensors = {}
        bands, start = [], 0
        for name, shape, dt, fill, off, nbytes in spans:
            bands.append(torch.arange(start, off))                    # the bytes between two tensors
            start = off + nbytes
            t = self.buf[off:off + nbytes].view(dt).view(*shape)
            t.fill_(fill)
            self.tensors[name] = t
        bands.append(torch.arange(start, at))
        self.guard_idx = torch.cat(bands).cuda()
        self.names = [(off, off + nbytes, name) for name, _, _, _, off, nbytes in spans]

    def check(self):
        bad = torch.nonzero(self.buf[self.guard_idx] != PATTERN)
        if bad.numel():
            pos = int(self.guard_idx[bad[0, 0]])
            near = min(self.names, key=lambda n: min(abs(pos - n[0]), abs(pos - n[1])))
            raise AssertionError(f"guard byte {pos} changed: a write outside output '{near[2]}' "
                                 f"(bytes {near[0]}..{near[1]})")


_LIVE = weakref.WeakSet()


def check_all_guards():
    """Every Dev that is alive: no output tensor was written outside its bounds."""
    torch.cuda.synchronize()
    for dev in list(_LIVE):
        dev.arena.check()


class Dev:
    """One layer's inputs and outputs in device memory.  Every tensor an entry point writes lives in a
    guarded arena (see Arena); the call wrappers below check the guards after each call."""

    def __init__(self, wl: W.Workload, k_blocks: bool = True, interleaved: bool = False):
        """interleaved: ONE pool [n_slots][2][S][d] (a slot's K tile and V tile next to each other)
        instead of two dense pools; k_pool / v_pool are then what the library is
        handed (v_pool = k_pool + one tile, tile_stride = 2 S d), k_tiles / v_tiles the [n_slots][S][d] views."""
        cfg = wl.cfg
        self.cfg, self.wl = cfg, wl
        self.tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        self.ctx_len = torch.from_numpy(wl.ctx_len).cuda()
        self.tile_stride = 2 * cfg.S * cfg.d if interleaved else 0
        self.p = B.make_problem(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.S, B.F32 if cfg.dtype == "f32" else B.BF16,
                                cfg.max_blocks, cfg.k, self.ctx_len, 0.0, tile_stride=self.tile_stride)
        self.q = to_dev(wl.q)
        self.n_slots = wl.n_slots
        if interleaved:
            kd, vd = to_dev(wl.k_pool), to_dev(wl.v_pool)
            self.kv_pool = torch.empty(kd.shape[0], 2, cfg.S, cfg.d, dtype=kd.dtype, device="cuda")
            self.kv_pool[:, 0], self.kv_pool[:, 1] = kd, vd
            flat = self.kv_pool.view(-1)
            self.k_pool, self.v_pool = flat, flat[cfg.S * cfg.d:]
            self.k_tiles, self.v_tiles = self.kv_pool[:, 0], self.kv_pool[:, 1]
        else:
            self.k_pool = to_dev(wl.k_pool)
            self.v_pool = to_dev(wl.v_pool)
            self.k_tiles, self.v_tiles = self.k_pool, self.v_pool
        pairs = (cfg.B, cfg.Hkv)
        if k_blocks:
            kb = np.full((cfg.B, cfg.Hkv, cfg.max_blocks, cfg.S, cfg.d), W._GARBAGE[cfg.dtype],
                         dtype=wl.k_pool.dtype)
            for (b, g) in wl.K:
                kb[b, g, :cfg.nb(b)] = wl.blocks_padded(b, g, "K")
            self.k_blocks = to_dev(kb)
        f32, i32, nan, ninf = torch.float32, torch.int32, float("nan"), float("-inf")
        lists, heads = (*pairs, cfg.k), (cfg.B, cfg.Hq)
        self.arena = Arena([
            ("digest", (*pairs, cfg.max_blocks, 2, cfg.d), self.tdt, 0),
            ("scores", (*pairs, cfg.max_blocks), f32, nan),
            ("sel_all", lists, i32, -7), ("sel_gpu", lists, i32, -7), ("slot_gpu", lists, i32, -7),
            ("sel_host", lists, i32, -7), ("n_gpu", pairs, i32, -7), ("n_host", pairs, i32, -7),
            ("o", (*heads, cfg.d), f32, nan), ("m", heads, f32, nan), ("l", heads, f32, nan),
            ("host_o", (*heads, cfg.d), f32, 0), ("host_m", heads, f32, ninf), ("host_l", heads, f32, 0),
            ("out", (*heads, cfg.d), self.tdt, 0), ("lse", heads, f32, nan),
            ("recall_blk", lists, i32, -7), ("recall_slot", lists, i32, -7), ("evict_blk", lists, i32, -7),
            ("n_recall", pairs, i32, -7),
            ("block_table", (*pairs, cfg.max_blocks), i32, -1),
            ("ws", (B.workspace_bytes(self.p),), torch.uint8, 0),
        ])
        for name, t in self.arena.tensors.items():
            setattr(self, name, t)
        self.block_table.copy_(torch.from_numpy(wl.block_table))
        _LIVE.add(self)

    # ---- the calls, one per boundary entry point
    def check_guards(self):
        if torch.cuda.is_current_stream_capturing():      # a call being recorded into a graph has not run
            return
        torch.cuda.synchronize()
        self.arena.check()

    def build_digests(self):
        B.build_digests(self.p, self.k_blocks, self.digest)
        self.check_guards()

    def score(self, q=None):
        B.score_blocks(self.p, self.q if q is None else q, self.digest, self.scores, self.ws)
        self.check_guards()

    def select(self, scores=None):
        B.select_topk(self.p, self.scores if scores is None else scores, self.block_table, self.sel_all,
                      self.sel_gpu, self.slot_gpu, self.n_gpu, self.sel_host, self.n_host, self.ws)
        self.check_guards()

    def attn(self, q=None):
        B.sparse_decode_attn(self.p, self.q if q is None else q, self.k_pool, self.v_pool, self.n_slots,
                             self.sel_gpu, self.slot_gpu, self.n_gpu, self.o, self.m, self.l, self.ws)
        self.check_guards()

    def merge(self, host=True):
        if host:
            B.merge_partials(self.p, self.o, self.m, self.l, self.host_o, self.host_m, self.host_l, self.out,
                             self.lse)
        else:
            B.merge_partials(self.p, self.o, self.m, self.l, None, None, None, self.out, self.lse)
        self.check_guards()

    def layer_step(self, q=None, host=True):
        h = (self.host_o, self.host_m, self.host_l) if host else (None, None, None)
        B.layer_step(self.p, self.q if q is None else q, self.digest, self.block_table, self.k_pool, self.v_pool,
                     self.n_slots, *h, self.scores, self.sel_all, self.sel_gpu, self.slot_gpu, self.n_gpu,
                     self.sel_host, self.n_host, self.out, self.lse, self.ws)
        self.check_guards()

    def recall(self, q=None):
        B.periodic_recall(self.p, self.q if q is None else q, self.digest, self.block_table, self.recall_blk,
                          self.recall_slot, self.evict_blk, self.n_recall, self.ws)
        self.check_guards()

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
