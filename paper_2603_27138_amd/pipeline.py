"""Layer-ahead co-attention pipeline (Sec. 3.3, Algorithm 1) over the library's entry points.

While the GPU works on layer i, the blocks of layer i+1 are selected with the predicted query, the
selected blocks that live on the host are handed to the host-side worker threads, and the GPU goes
on with layer i: its own partial attention (real query) over the resident selected blocks, merged
with the host's partial that was started during layer i-1.  Every few steps, after a layer's attention,
the blocks that became important return from the host (Sec. 3.4): the plan is made on the GPU, the
host packs the planned tiles, a copy engine moves them and a small kernel puts them into the slots the
plan freed, all beside the following layers' work.  This module only sequences calls and
copies a few kilobytes of lists and partial results between host and device; every step of the
method runs in the HIP library (device side) or in the worker threads (host side).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional

import numpy as np
import torch

from . import binding as B
from . import host as H


@dataclass
class Layer:
    """Cache state of one layer.  Device: digest [B][Hkv][mb][2][d], block_table [B][Hkv][mb] i32,
    k_pool / v_pool [n_slots][S][d].  Host (pinned CPU tensors): k_blocks / v_blocks
    [B][Hkv][mb][S][d], every block by logical index."""
    digest: torch.Tensor
    block_table: torch.Tensor
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    n_slots: int
    k_blocks: torch.Tensor
    v_blocks: torch.Tensor


class _LayerBuffers:
    def __init__(self, Bn, Hq, Hkv, d, mb, k, tdt):
        dev = dict(device="cuda")
        i32 = dict(dtype=torch.int32, **dev)
        f32 = dict(dtype=torch.float32, **dev)
        pairs = (Bn, Hkv)
        self.scores = torch.empty(*pairs, mb, **f32)
        self.sel_all, self.sel_gpu, self.slot_gpu, self.sel_host = (torch.empty(*pairs, k, **i32) for _ in range(4))
        self.n_gpu, self.n_host = torch.empty(pairs, **i32), torch.empty(pairs, **i32)
        self.ho, self.hm, self.hl = torch.empty(Bn, Hq, d, **f32), torch.empty(Bn, Hq, **f32), torch.empty(Bn, Hq, **f32)
        self.out = torch.empty(Bn, Hq, d, dtype=tdt, **dev)
        self.lse = torch.empty(Bn, Hq, **f32)
        pin = dict(pin_memory=True)
        self.sel_host_h = torch.empty(*pairs, k, dtype=torch.int32, **pin)
        self.n_host_h = torch.empty(pairs, dtype=torch.int32, **pin)
        self.q_pred_h = torch.empty(Bn, Hq, d, dtype=tdt, **pin)
        self.ho_h = torch.empty(Bn, Hq, d, dtype=torch.float32, **pin)
        self.hm_h = torch.empty(Bn, Hq, dtype=torch.float32, **pin)
        self.hl_h = torch.empty(Bn, Hq, dtype=torch.float32, **pin)
        self.selected = torch.cuda.Event()
        # periodic recall: the plan (device, and the part the host needs in pinned memory)
        self.recall_blk, self.recall_slot, self.evict_blk = (torch.empty(*pairs, k, **i32) for _ in range(3))
        self.n_recall = torch.empty(pairs, **i32)
        self.recall_blk_h = torch.empty(*pairs, k, dtype=torch.int32, **pin)
        self.n_recall_h = torch.empty(pairs, dtype=torch.int32, **pin)
        self.planned = torch.cuda.Event()
        self.arrived: Optional[torch.cuda.Event] = None   # set while recalled tiles are on their way


class LayerAheadPipeline:
    def __init__(self, Bn, Hq, Hkv, d, S, dtype, max_blocks, k, ctx_len: torch.Tensor, layers: List[Layer],
                 n_threads: int, filler: Optional[Callable[[int], None]] = None, recall_every: int = 0,
                 n_stage_threads: int = 2, max_recall_tiles: Optional[int] = None):
        """ctx_len: device int32 [B].  filler(i), if given, enqueues the rest of layer i's GPU work
        (projections, feed-forward) on the current stream, so that the host has the window the
        paper's method counts on.  recall_every = R > 0: after the attention of every step t with
        t % R == R - 1, each layer recalls (Sec. 3.4); max_recall_tiles bounds the staging buffers
        (default: every pair recalls its whole budget)."""
        self.layers = layers
        self.p = B.make_problem(Bn, Hq, Hkv, d, S, dtype, max_blocks, k, ctx_len, 0.0)
        self.hp = H.HostProblem(Bn, Hq, Hkv, d, S, dtype, max_blocks, k, 0.0)
        self.ctx_len = ctx_len
        self.ctx_len_h = ctx_len.cpu().numpy().copy()
        self.ws = B.alloc_workspace(self.p)
        tdt = torch.float32 if dtype == B.F32 else torch.bfloat16
        self.buf = [_LayerBuffers(Bn, Hq, Hkv, d, max_blocks, k, tdt) for _ in layers]
        self.worker = H.HostWorker(n_threads)
        self.filler = filler
        self.recall_every, self.step_no = int(recall_every), 0
        self.recalled_tiles = 0               # tiles moved by the last step's recalls
        if self.recall_every > 0:
            self.stager = H.HostWorker(n_stage_threads)   # a pool of its own: packing never waits for attention jobs
            self.copy_stream = torch.cuda.Stream()
            tiles = max(1, Bn * Hkv * k if max_recall_tiles is None else int(max_recall_tiles))
            self.staged_h = torch.empty(tiles, 2, S, d, dtype=tdt, pin_memory=True)
            self.staged = torch.empty(tiles, 2, S, d, dtype=tdt, device="cuda")
            self.tile_off_h = torch.zeros(max(1, Bn * Hkv), dtype=torch.int32, pin_memory=True)
            self.tile_off = torch.zeros(max(1, Bn * Hkv), dtype=torch.int32, device="cuda")
            self.staged_read = torch.cuda.Event()         # the copy engine is done with the pinned buffers
            self.staged_read.record()
        self.host_seconds: List[float] = []   # per layer: submit -> completion of the host's job
        self.wait_seconds: List[float] = []   # per layer: how long the enqueueing thread sat in wait()

    def close(self):
        self.worker.close()
        if self.recall_every > 0:
            self.stager.close()

    # -- Algorithm 1, "trigger next layer's CPU-side pre-computation"
    def _trigger(self, i: int, q_pred: torch.Tensor):
        L, b = self.layers[i], self.buf[i]
        B.score_blocks(self.p, q_pred, L.digest, b.scores, self.ws)
        B.select_topk(self.p, b.scores, L.block_table, b.sel_all, b.sel_gpu, b.slot_gpu, b.n_gpu, b.sel_host,
                      b.n_host, self.ws)
        b.sel_host_h.copy_(b.sel_host, non_blocking=True)
        b.n_host_h.copy_(b.n_host, non_blocking=True)
        b.q_pred_h.copy_(q_pred, non_blocking=True)
        b.selected.record()

    def _spawn(self, i: int):
        L, b = self.layers[i], self.buf[i]
        b.selected.synchronize()
        qh = b.q_pred_h.view(torch.int16) if b.q_pred_h.dtype == torch.bfloat16 else b.q_pred_h
        self.worker.submit(self.hp, qh, L.k_blocks, L.v_blocks, b.sel_host_h, b.n_host_h, self.ctx_len_h,
                           b.ho_h, b.hm_h, b.hl_h)

    # -- Algorithm 1, "compute current layer's attention" and "merge"
    def _attend(self, i: int, q: torch.Tensor):
        L, b = self.layers[i], self.buf[i]
        if b.arrived is not None:             # tiles recalled after this layer's last attention
            torch.cuda.current_stream().wait_event(b.arrived)
            b.arrived = None
        # the per-split partials stay in the workspace until _merge folds them together with the host's
        B.attn_partials(self.p, q, L.k_pool, L.v_pool, L.n_slots, b.sel_gpu, b.slot_gpu, b.n_gpu, self.ws)

    def _merge(self, i: int):
        b = self.buf[i]
        b.ho.copy_(b.ho_h, non_blocking=True)
        b.hm.copy_(b.hm_h, non_blocking=True)
        b.hl.copy_(b.hl_h, non_blocking=True)
        B.attn_finish(self.p, b.ho, b.hm, b.hl, b.out, b.lse, self.ws)

    # -- Sec. 3.4: plan on the GPU (the table changes at once, in stream order) ...
    def _plan_recall(self, i: int, q: torch.Tensor):
        L, b = self.layers[i], self.buf[i]
        B.periodic_recall(self.p, q, L.digest, L.block_table, b.recall_blk, b.recall_slot, b.evict_blk,
                          b.n_recall, self.ws)
        b.recall_blk_h.copy_(b.recall_blk, non_blocking=True)
        b.n_recall_h.copy_(b.n_recall, non_blocking=True)
        b.planned.record()

    # ... then the tiles: packed by the host, moved by a copy engine, placed by recall_scatter, all on
    # the copy stream; the layer's next attention waits for `arrived`
    def _move_recall(self, i: int):
        L, b = self.layers[i], self.buf[i]
        b.planned.synchronize()
        self.staged_read.synchronize()
        sh = self.staged_h.view(torch.int16) if self.staged_h.dtype == torch.bfloat16 else self.staged_h
        tiles = self.stager.stage_recall(self.hp, L.k_blocks, L.v_blocks, b.recall_blk_h, b.n_recall_h, sh,
                                         self.tile_off_h)
        self.stager.wait()
        self.recalled_tiles += tiles
        if tiles == 0:
            return
        with torch.cuda.stream(self.copy_stream):
            self.staged[:tiles].copy_(self.staged_h[:tiles], non_blocking=True)
            self.tile_off.copy_(self.tile_off_h, non_blocking=True)
            self.staged_read.record()
            B.recall_scatter(self.p, self.staged, self.tile_off, b.recall_blk, b.recall_slot, b.n_recall,
                             L.k_pool, L.v_pool, L.n_slots)
            b.arrived = torch.cuda.Event()
            b.arrived.record()

    def step(self, qs: List[torch.Tensor], q_preds: List[torch.Tensor], host: bool = True):
        """One decode step over all layers.  qs[i]: the real query of layer i, q_preds[i]: the one
        predicted a layer ahead.  host=False leaves the host worker out (its partials are taken as
        they stand in the pinned buffers): the GPU-only reference for the idle share."""
        import time
        n = len(self.layers)
        self.host_seconds, self.wait_seconds = [], []
        due = self.recall_every > 0 and self.step_no % self.recall_every == self.recall_every - 1
        self.recalled_tiles = 0
        pending = None                        # layer whose plan is made and whose tiles are still to move
        self._trigger(0, q_preds[0])
        if host:
            self._spawn(0)
        for i in range(n):
            if i + 1 < n:
                self._trigger(i + 1, q_preds[i + 1])
            self._attend(i, qs[i])
            if self.filler is not None:
                self.filler(i)
            # Algorithm 1 spawns the host's job for layer i+1 as soon as its blocks are chosen, beside
            # this layer's GPU attention: here, once this layer's GPU work is queued (the enqueueing
            # thread then waits for the selection, which the GPU finished before it began the attention).
            # The worker takes the job behind the one of layer i if that is still running.
            if host and i + 1 < n:
                self._spawn(i + 1)
            if pending is not None:           # the GPU has this layer's work queued: now see to the last one's tiles
                self._move_recall(pending)
                pending = None
            if host:
                t0 = time.perf_counter()
                self.host_seconds.append(self.worker.wait())      # the oldest job: layer i's
                self.wait_seconds.append(time.perf_counter() - t0)
            self._merge(i)
            if due:
                self._plan_recall(i, qs[i])
                pending = i
        if pending is not None:
            self._move_recall(pending)
        self.step_no += 1
        return [b.out for b in self.buf]
