"""Seeded synthetic decode-attention workloads.

Input plumbing only: random draws, planting, residency maps, paging into the
KV pool and storage-type conversion.  None of the method's arithmetic (digest,
score, selection, attention, merge, recall) lives here; both the HIP path and
the CPU oracle consume what this module produces.

The inputs stand in for the Qwen3 decode workloads of the paper's evaluation
(Sec. 4.3: budget 2048, block 32): standard-normal keys and values, a few
"heavy" blocks whose keys are shifted along the direction of the summed query
of the head group so that selection is neither trivial nor uniform, a fixed
fraction of blocks marked host-resident, shuffled pool slots so reads are
genuinely paged.

Storage types: "f32" arrays are numpy float32; "bf16" arrays are numpy uint16
holding the upper 16 bits of the binary32 pattern (round-to-nearest-even).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20260327

# ---------------------------------------------------------------- storage types


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to bf16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f32(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.float32:
        return a
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    raise TypeError(a.dtype)


# ---------------------------------------------------------------- configuration


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    S: int
    dtype: str                 # "f32" | "bf16"
    ctx: Tuple[int, ...]       # tokens per sequence, len B
    k: int                     # block budget per (sequence, KV head)
    planted: float             # >=1: that many blocks per pair; <1: fraction of the pair's blocks
    p_host: float              # fraction of each pair's blocks kept in host memory
    seed: int
    recall_interval: int = 0   # 0: no periodic recall
    steps: int = 1
    layers: int = 1
    rho: float = 0.90          # step-to-step query correlation: ~12 % of the top-k set changes per step

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def max_blocks(self) -> int:
        return max((c + self.S - 1) // self.S for c in self.ctx) if self.ctx else 0

    def nb(self, b: int) -> int:
        return (self.ctx[b] + self.S - 1) // self.S

    @property
    def sm_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))


def tiny() -> Config:
    """Config 1: batch 1, GQA 4, d 64, fp32, 2048 tokens in 128 blocks of 16, k = 16."""
    return Config("C1-tiny", 1, 4, 1, 64, 16, "f32", (2048,), 16, 8, 0.0, BASE_SEED + 1)


def qwen3_8b(B: int = 8, ctx: int = 32768) -> Config:
    """Config 2: 32 q / 8 KV heads, d 128, bf16, block 32, k = 64, 40 % host-resident."""
    return Config("C2-qwen3-8b", B, 32, 8, 128, 32, "bf16", (ctx,) * B, 64, 0.05, 0.40, BASE_SEED + 2)


def qwen3_32b(B: int = 16, ctx: int = 32768) -> Config:
    """Config 3: 64 q / 8 KV heads (GQA 8), d 128, bf16, block 32, k = 64, 50 % host-resident."""
    return Config("C3-qwen3-32b", B, 64, 8, 128, 32, "bf16", (ctx,) * B, 64, 0.05, 0.50, BASE_SEED + 3)


def long_context(B: int = 4, ctx: int = 131072, steps: int = 32) -> Config:
    """Config 4: 131072 tokens in 4096 blocks, k = 128, 75 % host, recall every 8 steps."""
    return Config("C4-long", B, 64, 8, 128, 32, "bf16", (ctx,) * B, 128, 0.05, 0.75, BASE_SEED + 4,
                  recall_interval=8, steps=steps)


def full_step(B: int = 32, layers: int = 64, lo: int = 4096, hi: int = 65536, steps: int = 32) -> Config:
    """Config 5: ragged contexts uniform in [lo, hi] rounded to blocks of 32, k = 64, recall every 16."""
    rng = np.random.default_rng([BASE_SEED + 5, 7])
    ctx = tuple(int(32 * rng.integers(lo // 32, hi // 32, endpoint=True)) for _ in range(B))
    return Config("C5-full-step", B, 64, 8, 128, 32, "bf16", ctx, 64, 0.05, 0.50, BASE_SEED + 5,
                  recall_interval=16, steps=steps, layers=layers)


def shrink(cfg: Config, **kw) -> Config:
    """A reduced copy of a config (for cases the oracle finishes in seconds)."""
    return replace(cfg, **kw)


# ---------------------------------------------------------------- generation

_STREAM_Q, _STREAM_KV, _STREAM_PLANT, _STREAM_HOST, _STREAM_SLOT, _STREAM_DRIFT = range(6)


def gen_q(cfg: Config, layer: int = 0, step: int = 0) -> np.ndarray:
    """Query [B][Hq][d] in storage type.  Steps > 0 drift: q <- rho q + sqrt(1-rho^2) eps."""
    out = np.empty((cfg.B, cfg.Hq, cfg.d), dtype=np.float32)
    for b in range(cfg.B):
        rng = np.random.default_rng([cfg.seed, layer, b, _STREAM_Q])
        q = rng.standard_normal((cfg.Hq, cfg.d), dtype=np.float32)
        if step > 0:
            drng = np.random.default_rng([cfg.seed, layer, b, _STREAM_DRIFT])
            a, c = np.float32(cfg.rho), np.float32(np.sqrt(1.0 - cfg.rho * cfg.rho))
            for _ in range(step):
                q = a * q + c * drng.standard_normal((cfg.Hq, cfg.d), dtype=np.float32)
        out[b] = q
    return to_storage(out, cfg.dtype)


def gen_q_pred(q: np.ndarray, cos: float, seed: int) -> np.ndarray:
    """A stand-in for the query predicted one layer ahead (Sec. 3.3): per head, a vector of the same
    norm as the real query at cosine similarity `cos` to it (the paper's table reports 0.93-0.97).
    q: [B][Hq][d] storage array; returns the same shape and type."""
    qf = storage_to_f32(q).astype(np.float64)
    rng = np.random.default_rng([int(seed), 77])
    n = rng.standard_normal(qf.shape)
    qn = np.linalg.norm(qf, axis=-1, keepdims=True)
    qn = np.where(qn > 0, qn, 1.0)
    n -= (n * qf).sum(-1, keepdims=True) / (qn * qn) * qf          # the part orthogonal to q
    n *= qn / np.linalg.norm(n, axis=-1, keepdims=True)            # same norm as q
    out = cos * qf + np.sqrt(max(0.0, 1.0 - cos * cos)) * n
    return to_storage(out.astype(np.float32), "bf16" if q.dtype == np.uint16 else "f32")


def _n_planted(cfg: Config, nb: int) -> int:
    n = int(cfg.planted) if cfg.planted >= 1 else int(round(cfg.planted * nb))
    return min(n, nb)


def gen_pair(cfg: Config, layer: int, b: int, g: int, q0: np.ndarray):
    """Keys/values of one (sequence, KV head) pair.

    q0: the step-0 query [B][Hq][d] in storage type (planting is aligned to it).
    Returns (K, V, planted_ids): K, V are logical [ctx_len][d] storage arrays.
    """
    ctx, S, d, G = cfg.ctx[b], cfg.S, cfg.d, cfg.G
    nb = cfg.nb(b)
    rng = np.random.default_rng([cfg.seed, layer, b, g, _STREAM_KV])
    K = rng.standard_normal((ctx, d), dtype=np.float32)
    V = rng.standard_normal((ctx, d), dtype=np.float32)
    prng = np.random.default_rng([cfg.seed, layer, b, g, _STREAM_PLANT])
    planted = np.sort(prng.permutation(nb)[: _n_planted(cfg, nb)]).astype(np.int32)
    qg = storage_to_f32(q0[b, g * G:(g + 1) * G]).astype(np.float64).sum(axis=0)
    u = (qg / max(np.linalg.norm(qg), 1e-30)).astype(np.float32)
    for j in planted:
        K[j * S:min(ctx, (j + 1) * S)] += np.float32(3.0) * u
    return to_storage(K, cfg.dtype), to_storage(V, cfg.dtype), planted


def gen_block_table(cfg: Config, layer: int = 0):
    """Residency map [B][Hkv][max_blocks] (pool slot, or -1 for host / beyond the context).

    Each pair keeps exactly round(p_host * nb) blocks in host memory, chosen by
    a seeded permutation independent of planting; resident blocks get distinct
    slots and the slot order is one global seeded shuffle.  Returns (table, n_slots).
    """
    table = np.full((cfg.B, cfg.Hkv, cfg.max_blocks), -1, dtype=np.int32)
    resident = []
    for b in range(cfg.B):
        nb = cfg.nb(b)
        for g in range(cfg.Hkv):
            rng = np.random.default_rng([cfg.seed, layer, b, g, _STREAM_HOST])
            n_host = int(round(cfg.p_host * nb))
            ids = np.sort(rng.permutation(nb)[n_host:])
            resident.append((b, g, ids))
    n_slots = int(sum(len(r[2]) for r in resident))
    srng = np.random.default_rng([cfg.seed, layer, _STREAM_SLOT])
    slots = srng.permutation(n_slots).astype(np.int32)
    at = 0
    for b, g, ids in resident:
        table[b, g, ids] = slots[at:at + len(ids)]
        at += len(ids)
    return table, n_slots


# Tail rows of a partially filled last block are never valid tokens; they are
# filled with this pattern (a NaN in either storage type) so that a kernel that
# lets them leak into a result is caught.
_GARBAGE = {"f32": np.float32(np.nan), "bf16": np.uint16(0x7FC1)}


@dataclass
class Workload:
    cfg: Config
    layer: int
    q: np.ndarray                      # [B][Hq][d] storage, step 0
    ctx_len: np.ndarray                # int32 [B]
    K: Dict[Tuple[int, int], np.ndarray] = field(default_factory=dict)   # logical, per pair
    V: Dict[Tuple[int, int], np.ndarray] = field(default_factory=dict)
    planted: Dict[Tuple[int, int], np.ndarray] = field(default_factory=dict)
    block_table: Optional[np.ndarray] = None
    n_slots: int = 0
    k_pool: Optional[np.ndarray] = None   # [n_slots][S][d] storage
    v_pool: Optional[np.ndarray] = None

    def blocks_padded(self, b: int, g: int, which: str) -> np.ndarray:
        """The pair's K or V as [nb][S][d], tail of the last block filled with garbage."""
        cfg = self.cfg
        a = (self.K if which == "K" else self.V)[(b, g)]
        nb = cfg.nb(b)
        if a.shape[0] == nb * cfg.S:
            return a.reshape(nb, cfg.S, cfg.d)
        full = np.full((nb * cfg.S, cfg.d), _GARBAGE[cfg.dtype], dtype=a.dtype)
        full[: a.shape[0]] = a
        return full.reshape(nb, cfg.S, cfg.d)


def pack_pool(wl: Workload, table: np.ndarray, n_slots: int):
    """Page the resident blocks of every pair into [n_slots][S][d] K and V pools."""
    cfg = wl.cfg
    sdt = np.float32 if cfg.dtype == "f32" else np.uint16
    k_pool = np.full((max(n_slots, 1), cfg.S, cfg.d), _GARBAGE[cfg.dtype], dtype=sdt)
    v_pool = np.full((max(n_slots, 1), cfg.S, cfg.d), _GARBAGE[cfg.dtype], dtype=sdt)
    for (b, g) in wl.K:
        nb = cfg.nb(b)
        row = table[b, g, :nb]
        ids = np.nonzero(row >= 0)[0]
        if len(ids) == 0:
            continue
        k_pool[row[ids]] = wl.blocks_padded(b, g, "K")[ids]
        v_pool[row[ids]] = wl.blocks_padded(b, g, "V")[ids]
    return k_pool, v_pool


def generate(cfg: Config, layer: int = 0, pairs: Optional[Sequence[Tuple[int, int]]] = None,
             with_pool: bool = True, workers: int = 8) -> Workload:
    """Build the step-0 workload of one layer.

    pairs: restrict K/V generation to these (b, g) pairs (any pair can be
    regenerated on its own: each has its own random stream).  The pool is only
    built when every pair is generated.
    """
    q = gen_q(cfg, layer, 0)
    wl = Workload(cfg, layer, q, np.asarray(cfg.ctx, dtype=np.int32))
    todo = list(pairs) if pairs is not None else [(b, g) for b in range(cfg.B) for g in range(cfg.Hkv)]

    def one(p):
        return p, gen_pair(cfg, layer, p[0], p[1], q)

    if workers > 1 and len(todo) > 1:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            results = list(ex.map(one, todo))
    else:
        results = [one(p) for p in todo]
    for p, (K, V, planted) in results:
        wl.K[p], wl.V[p], wl.planted[p] = K, V, planted
    wl.block_table, wl.n_slots = gen_block_table(cfg, layer)
    if with_pool and pairs is None:
        wl.k_pool, wl.v_pool = pack_pool(wl, wl.block_table, wl.n_slots)
    return wl
