"""CPU oracle (test infrastructure).

A thin ctypes/numpy layer over ``scout_oracle.c``: it loops over (sequence, KV
head) pairs and query heads and calls the per-pair C functions, nothing more.
Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the product package never does, and this package imports nothing of
the product.

Storage types: ``float32`` arrays are passed as they are; bf16 data is carried
as ``uint16`` arrays holding the upper half of the binary32 pattern.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scout_oracle.c")
# SCOUT_ORACLE_LIB names another build of the same source (the tests' sanitizer build) to load instead
_LIB = os.environ.get("SCOUT_ORACLE_LIB") or os.path.join(_HERE, "libscout_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no fast-math). Returns the library path."""
    if os.environ.get("SCOUT_ORACLE_LIB"):
        return _LIB
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, ip, dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.orc_num_blocks.argtypes = [ci, ci]
        lib.orc_num_blocks.restype = ci
        lib.orc_digest.argtypes = [ci, vp, ci, ci, ci, vp]
        lib.orc_digest.restype = None
        lib.orc_score.argtypes = [ci, vp, vp, ci, ci, ci, dp]
        lib.orc_score.restype = None
        lib.orc_rank.argtypes = [dp, ci, ip]
        lib.orc_rank.restype = None
        lib.orc_select.argtypes = [dp, ci, ci, ip]
        lib.orc_select.restype = ci
        lib.orc_split.argtypes = [ip, ci, ip, ci, ip, ip, ip, ip]
        lib.orc_split.restype = None
        lib.orc_partial_attn.argtypes = [ci, vp, vp, vp, ip, ci, ci, ci, ci, cd, dp, dp, dp]
        lib.orc_partial_attn.restype = None
        lib.orc_merge.argtypes = [dp, cd, cd, dp, cd, cd, ci, dp, dp]
        lib.orc_merge.restype = None
        lib.orc_recall_plan.argtypes = [dp, ci, ci, ip, ip, ip, ip]
        lib.orc_recall_plan.restype = ci
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"storage arrays must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _vp(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _ip(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def _dp(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_blocks(ctx_len: int, S: int) -> int:
    return _L().orc_num_blocks(int(ctx_len), int(S))


def digest(K: np.ndarray, ctx_len: int, S: int) -> np.ndarray:
    """K: [>=ctx_len][d] storage array of one pair. Returns [nb][2][d] (min, max)."""
    K = np.ascontiguousarray(K)
    d = K.shape[1]
    nb = num_blocks(ctx_len, S)
    out = np.zeros((nb, 2, d), dtype=K.dtype)
    _L().orc_digest(_dtype_code(K), _vp(K), int(ctx_len), int(S), int(d), _vp(out))
    return out


def score(q: np.ndarray, dig: np.ndarray) -> np.ndarray:
    """q: [G][d], dig: [nb][2][d] (same storage type). Returns float64 [nb]."""
    q = np.ascontiguousarray(q)
    dig = np.ascontiguousarray(dig)
    assert q.dtype == dig.dtype
    G, d = q.shape
    nb = dig.shape[0]
    s = np.zeros(nb, dtype=np.float64)
    _L().orc_score(_dtype_code(q), _vp(q), _vp(dig), nb, G, d, _dp(s))
    return s


def digest_sum(K: np.ndarray, ctx_len: int, S: int) -> np.ndarray:
    """Mean-pooled digest stored as binary32 sums of the valid keys of each block: float32 [nb][d]."""
    K = np.ascontiguousarray(K)
    d = K.shape[1]
    nb = (int(ctx_len) + S - 1) // S
    out = np.zeros((nb, d), dtype=np.float32)
    L = _L()
    L.orc_digest_sum.restype = None
    L.orc_digest_sum.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    L.orc_digest_sum(_dtype_code(K), K.ctypes.data, int(ctx_len), int(S), d, out.ctypes.data)
    return out


def append_sum(S: int, ctx_len: int, k_new: np.ndarray, sums: np.ndarray) -> None:
    """The token at position ctx_len joins the sums [max_blocks][d] (float32, updated in place)."""
    k_new = np.ascontiguousarray(k_new)
    assert sums.dtype == np.float32 and sums.flags["C_CONTIGUOUS"] and sums.shape[1] == k_new.shape[-1]
    L = _L()
    L.orc_append_sum.restype = None
    L.orc_append_sum.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 2
    L.orc_append_sum(_dtype_code(k_new), int(S), sums.shape[1], sums.shape[0], int(ctx_len), k_new.ctypes.data,
                     sums.ctypes.data)


def score_mean(q: np.ndarray, sums: np.ndarray, ctx_len: int, S: int) -> np.ndarray:
    """q: [G][d] storage, sums: float32 [nb][d].  Returns float64 [nb]: sum over heads of q . mean."""
    q = np.ascontiguousarray(q)
    sums = np.ascontiguousarray(sums, dtype=np.float32)
    G, d = q.shape
    nb = sums.shape[0]
    s = np.zeros(nb, dtype=np.float64)
    L = _L()
    L.orc_score_mean.restype = None
    L.orc_score_mean.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 5 + [ctypes.c_void_p]
    L.orc_score_mean(_dtype_code(q), q.ctypes.data, sums.ctypes.data, nb, G, d, int(ctx_len), int(S), s.ctypes.data)
    return s


def decision_scores(s: np.ndarray) -> np.ndarray:
    """Scores as the selection sees them: rounded once to binary32.

    The boundary carries scores as binary32, so both sides take the top-k
    decision on the binary32 value.
    """
    return s.astype(np.float32).astype(np.float64)


def rank(s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, dtype=np.float64)
    r = np.zeros(len(s), dtype=np.int32)
    _L().orc_rank(_dp(s), len(s), _ip(r))
    return r


def select(s: np.ndarray, k: int) -> np.ndarray:
    """Returns int32 [k]: the k_eff selected block indices ascending, then -1."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    sel = np.full(max(k, 1), -1, dtype=np.int32)
    _L().orc_select(_dp(s), len(s), int(k), _ip(sel))
    return sel[:k]


def split(sel: np.ndarray, table: np.ndarray):
    """sel: [k] padded with -1; table: [>=nb] slots. Returns (sel_gpu, n_gpu, sel_host, n_host)."""
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    table = np.ascontiguousarray(table, dtype=np.int32)
    k = len(sel)
    n_sel = int((sel >= 0).sum())
    sg = np.full(max(k, 1), -1, dtype=np.int32)
    sh = np.full(max(k, 1), -1, dtype=np.int32)
    ng, nh = ctypes.c_int(0), ctypes.c_int(0)
    _L().orc_split(_ip(sel), n_sel, _ip(table), k, _ip(sg), ctypes.byref(ng), _ip(sh), ctypes.byref(nh))
    return sg[:k], ng.value, sh[:k], nh.value


def partial_attn(q_h: np.ndarray, K: np.ndarray, V: np.ndarray, blocks, ctx_len: int, S: int,
                 sm_scale: float):
    """One head over the listed blocks. Returns (o float64 [d], m, l)."""
    q_h = np.ascontiguousarray(q_h)
    K = np.ascontiguousarray(K)
    V = np.ascontiguousarray(V)
    assert q_h.dtype == K.dtype == V.dtype
    d = K.shape[1]
    blocks = np.ascontiguousarray(np.asarray(blocks, dtype=np.int32))
    blocks = blocks[blocks >= 0]
    blk = blocks if len(blocks) else np.zeros(1, dtype=np.int32)
    o = np.zeros(d, dtype=np.float64)
    m, l = ctypes.c_double(0), ctypes.c_double(0)
    _L().orc_partial_attn(_dtype_code(K), _vp(q_h), _vp(K), _vp(V), _ip(blk), len(blocks),
                          int(ctx_len), int(S), int(d), float(sm_scale), _dp(o),
                          ctypes.byref(m), ctypes.byref(l))
    return o, m.value, l.value


def merge(o_a, m_a, l_a, o_b, m_b, l_b):
    """Returns (out float64 [d], lse)."""
    o_a = np.ascontiguousarray(o_a, dtype=np.float64)
    o_b = np.ascontiguousarray(o_b, dtype=np.float64)
    d = len(o_a)
    out = np.zeros(d, dtype=np.float64)
    lse = ctypes.c_double(0)
    _L().orc_merge(_dp(o_a), float(m_a), float(l_a), _dp(o_b), float(m_b), float(l_b), d,
                   _dp(out), ctypes.byref(lse))
    return out, lse.value


def recall_plan(s: np.ndarray, k: int, table: np.ndarray):
    """table is updated in place. Returns (recall_blk, recall_slot, evict_blk, n)."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    assert table.dtype == np.int32 and table.flags["C_CONTIGUOUS"]
    rb = np.full(max(k, 1), -1, dtype=np.int32)
    rs = np.full(max(k, 1), -1, dtype=np.int32)
    eb = np.full(max(k, 1), -1, dtype=np.int32)
    n = _L().orc_recall_plan(_dp(s), len(s), int(k), _ip(table), _ip(rb), _ip(rs), _ip(eb))
    return rb[:k], rs[:k], eb[:k], n


def append(dtype: int, S: int, ctx_len: int, k_new: np.ndarray, v_new: np.ndarray, new_slot: int,
           dig: np.ndarray, table: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray,
           host_k: np.ndarray = None, host_v: np.ndarray = None) -> int:
    """Decode append for one pair; dig [max_blocks][2][d], table [max_blocks], the pools
    [n_slots][S][d] and (if given) the host's copy of every block [max_blocks][S][d] are updated
    in place.  Returns the new context length."""
    d = k_new.shape[-1]
    for a in (k_new, v_new, dig, k_pool, v_pool):
        assert a.flags["C_CONTIGUOUS"] and a.dtype == (np.float32 if dtype == F32 else np.uint16)
    assert table.dtype == np.int32 and table.flags["C_CONTIGUOUS"]
    assert dig.shape == (len(table), 2, d) and k_pool.shape[1:] == (S, d) and v_pool.shape == k_pool.shape
    hk = hv = None
    if host_k is not None:
        for a in (host_k, host_v):
            assert a.flags["C_CONTIGUOUS"] and a.dtype == k_new.dtype and a.shape == (len(table), S, d)
        hk, hv = host_k.ctypes.data, host_v.ctypes.data
    L = _L()
    L.orc_append.restype = ctypes.c_int
    L.orc_append.argtypes = ([ctypes.c_int] * 5 + [ctypes.c_void_p] * 2 + [ctypes.c_int] + [ctypes.c_void_p] * 4 +
                             [ctypes.c_long] + [ctypes.c_void_p] * 2)
    return L.orc_append(int(dtype), int(S), int(d), len(table), int(ctx_len), k_new.ctypes.data,
                        v_new.ctypes.data, int(new_slot), dig.ctypes.data, table.ctypes.data,
                        k_pool.ctypes.data, v_pool.ctypes.data, len(k_pool), hk, hv)


def recall_fetch(src_k: np.ndarray, src_v: np.ndarray, recall_blk, recall_slot, n: int,
                 k_pool: np.ndarray, v_pool: np.ndarray) -> int:
    """Copies the tiles a recall plan names from one pair's blocks [max_blocks][S][d] into the pools
    [n_slots][S][d] (updated in place).  Returns the number of tiles copied."""
    for a in (src_k, src_v, k_pool, v_pool):
        assert a.flags["C_CONTIGUOUS"] and a.dtype == src_k.dtype
    mb, S, d = src_k.shape
    assert src_v.shape == src_k.shape and k_pool.shape[1:] == (S, d) and v_pool.shape == k_pool.shape
    rb = np.ascontiguousarray(recall_blk, dtype=np.int32)
    rs = np.ascontiguousarray(recall_slot, dtype=np.int32)
    L = _L()
    L.orc_recall_fetch.restype = ctypes.c_int
    L.orc_recall_fetch.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p] * 4 + [ctypes.c_int] + [ctypes.c_void_p] * 2 + [ctypes.c_long]
    return L.orc_recall_fetch(_dtype_code(src_k), S, d, mb, src_k.ctypes.data, src_v.ctypes.data, rb.ctypes.data,
                              rs.ctypes.data, int(n), k_pool.ctypes.data, v_pool.ctypes.data, len(k_pool))


def recall_stage(src_k: np.ndarray, src_v: np.ndarray, recall_blk: np.ndarray, n_recall: np.ndarray):
    """Packs the tiles that the plans of all pairs name.  src_k / src_v are [pairs][max_blocks][S][d],
    recall_blk is [pairs][k], n_recall is [pairs].  Returns (staged [tiles][2][S][d], tile_off [pairs])."""
    pairs, mb, S, d = src_k.shape
    assert src_v.shape == src_k.shape and src_k.flags["C_CONTIGUOUS"] and src_v.flags["C_CONTIGUOUS"]
    rb = np.ascontiguousarray(recall_blk, dtype=np.int32)
    nr = np.ascontiguousarray(n_recall, dtype=np.int32)
    k = rb.shape[1]
    assert rb.shape == (pairs, k) and nr.shape == (pairs,)
    total = int(np.clip(nr, 0, k).sum())
    staged = np.zeros((total, 2, S, d), dtype=src_k.dtype)
    off = np.zeros(pairs, dtype=np.int32)
    L = _L()
    L.orc_recall_stage.restype = ctypes.c_long
    L.orc_recall_stage.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 6
    got = L.orc_recall_stage(_dtype_code(src_k), S, d, mb, k, pairs, src_k.ctypes.data, src_v.ctypes.data,
                             rb.ctypes.data, nr.ctypes.data, staged.ctypes.data, off.ctypes.data)
    assert got == total
    return staged, off


def recall_scatter(staged: np.ndarray, tile_off: np.ndarray, recall_blk: np.ndarray, recall_slot: np.ndarray,
                   n_recall: np.ndarray, max_blocks: int, k_pool: np.ndarray, v_pool: np.ndarray) -> int:
    """Puts staged tiles into the pools [n_slots][S][d] (updated in place).  Returns the number placed."""
    rb = np.ascontiguousarray(recall_blk, dtype=np.int32)
    rs = np.ascontiguousarray(recall_slot, dtype=np.int32)
    nr = np.ascontiguousarray(n_recall, dtype=np.int32)
    off = np.ascontiguousarray(tile_off, dtype=np.int32)
    pairs, k = rb.shape
    n_slots, S, d = k_pool.shape
    for a in (staged, k_pool, v_pool):
        assert a.flags["C_CONTIGUOUS"] and a.dtype == k_pool.dtype
    assert staged.shape[1:] == (2, S, d) and v_pool.shape == k_pool.shape and rs.shape == rb.shape
    L = _L()
    L.orc_recall_scatter.restype = ctypes.c_long
    L.orc_recall_scatter.argtypes = [ctypes.c_int] * 6 + [ctypes.c_void_p] * 7 + [ctypes.c_long]
    return L.orc_recall_scatter(_dtype_code(k_pool), S, d, int(max_blocks), k, pairs, staged.ctypes.data,
                                off.ctypes.data, rb.ctypes.data, rs.ctypes.data, nr.ctypes.data,
                                k_pool.ctypes.data, v_pool.ctypes.data, n_slots)


def force_blocks(s: np.ndarray, n_sink: int, n_tail: int) -> np.ndarray:
    """Scores with the first n_sink and the last n_tail blocks raised to +inf (a copy)."""
    out = np.ascontiguousarray(s, dtype=np.float64).copy()
    L = _L()
    L.orc_force_blocks.restype = None
    L.orc_force_blocks.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.orc_force_blocks(_dp(out), len(out), int(n_sink), int(n_tail))
    return out


def score_max(q: np.ndarray, dig: np.ndarray) -> np.ndarray:
    """As score(), with the maximum over the group's heads instead of their sum."""
    q = np.ascontiguousarray(q)
    dig = np.ascontiguousarray(dig)
    assert q.dtype == dig.dtype
    G, d = q.shape
    nb = dig.shape[0]
    s = np.zeros(nb, dtype=np.float64)
    L = _L()
    L.orc_score_max.restype = None
    L.orc_score_max.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                ctypes.POINTER(ctypes.c_double)]
    L.orc_score_max(_dtype_code(q), _vp(q), _vp(dig), nb, G, d, _dp(s))
    return s
