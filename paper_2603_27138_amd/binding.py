"""ctypes binding of libscout.so: argument marshalling only.

Every function takes torch CUDA tensors (device memory owned by the caller),
passes their addresses and the current HIP stream to the C ABI of
``include/scout.h`` and raises ``ScoutError`` on a negative return code.  There
is no CPU fallback: if the library has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscout.so")

F32, BF16 = 0, 1
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = ["scout_version", "scout_strerror", "scout_workspace_bytes", "build_digests", "append_token", "score_blocks",
           "select_topk", "sparse_decode_attn", "merge_partials", "periodic_recall", "recall_fetch", "recall_scatter",
           "scout_layer_step", "scout_set_attn_mode", "scout_attn_partials", "scout_attn_finish",
           "sparse_decode_attn_static"]
# measurement aids live in a library of their own (include/scout_calib.h)
CALIB_LIB_PATH = os.path.join(_HERE, "libscout_calib.so")
CALIB_EXPORTS = ["scout_calib_copy", "scout_calib_read", "scout_calib_gather"]


class ScoutError(RuntimeError):
    def __init__(self, fn: str, code: int, msg: str):
        super().__init__(f"{fn}: {msg} ({code})")
        self.code = code


class Problem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("S", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("k", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("n_sink", ctypes.c_int32), ("n_tail", ctypes.c_int32), ("group_max", ctypes.c_int32),
                ("per_head", ctypes.c_int32), ("digest_kind", ctypes.c_int32), ("tile_stride", ctypes.c_int32),
                ("ctx_len", ctypes.c_void_p)]


_lib = None


def lib():
    """The loaded shared library (built beforehand with ``paper_2603_27138_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2603_27138_amd.build); "
                "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
        pp = ctypes.POINTER(Problem)
        L.scout_version.restype = ctypes.c_int
        L.scout_strerror.restype = ctypes.c_char_p
        L.scout_strerror.argtypes = [ctypes.c_int]
        L.scout_set_attn_mode.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.scout_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.build_digests.argtypes = [pp, vp, vp, vp]
        L.append_token.argtypes = [pp] + [vp] * 8 + [i64, vp, vp, vp]
        L.score_blocks.argtypes = [pp, vp, vp, vp, vp, sz, vp]
        L.select_topk.argtypes = [pp] + [vp] * 9 + [sz, vp]
        L.sparse_decode_attn.argtypes = [pp, vp, vp, vp, i64] + [vp] * 7 + [sz, vp]
        L.sparse_decode_attn_static.argtypes = [pp, vp, vp, vp, i64] + [vp] * 6 + [vp]
        L.merge_partials.argtypes = [pp] + [vp] * 9
        L.periodic_recall.argtypes = [pp] + [vp] * 8 + [sz, vp]
        L.recall_fetch.argtypes = [pp] + [vp] * 7 + [i64, vp]
        L.recall_scatter.argtypes = [pp, vp, i64] + [vp] * 6 + [i64, vp]
        L.scout_attn_partials.argtypes = [pp, vp, vp, vp, i64] + [vp] * 4 + [sz, vp]
        L.scout_attn_finish.argtypes = [pp] + [vp] * 6 + [sz, vp]
        L.scout_layer_step.argtypes = [pp, vp, vp, vp, vp, vp, i64] + [vp] * 13 + [sz, vp]
        for name in EXPORTS:
            if name not in ("scout_strerror",):
                getattr(L, name).restype = getattr(L, name).restype or ctypes.c_int
        _lib = L
    return _lib


_calib = None


def calib_lib():
    """The measurement aids (copy of known size, bare stream, bare gather): benchmarks and profiling only."""
    global _calib
    if _calib is None:
        if not os.path.exists(CALIB_LIB_PATH):
            raise FileNotFoundError(f"{CALIB_LIB_PATH} is missing: build it first (python -m paper_2603_27138_amd.build)")
        L = ctypes.CDLL(CALIB_LIB_PATH)
        vp, sz, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
        L.scout_calib_copy.argtypes = [vp, vp, sz, vp]
        L.scout_calib_read.argtypes = [vp, sz, vp, vp]
        L.scout_calib_gather.argtypes = [ctypes.POINTER(Problem), vp, vp, i64, vp, vp, vp, vp]
        for name in CALIB_EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        _calib = L
    return _calib


def _check(fn: str, rc: int):
    if rc != 0:
        raise ScoutError(fn, rc, lib().scout_strerror(rc).decode())


_recording = None   # a Prepared being filled: calls are recorded instead of made


def _call(fn: str, cfunc, *cargs):
    if _recording is not None:
        _recording.calls.append((fn, cfunc, cargs))
        return
    _check(fn, cfunc(*cargs))


class Prepared:
    """Calls with their arguments already marshalled (pointers, sizes, stream): replaying them costs
    one foreign call each.  Valid while the tensors it was prepared with are alive and unmoved, on the
    stream that was current when it was prepared."""

    def __init__(self):
        self.calls = []

    def __call__(self):
        for fn, cfunc, cargs in self.calls:
            rc = cfunc(*cargs)
            if rc != 0:
                _check(fn, rc)


def prepare(fn, *args, **kw) -> Prepared:
    """Record the library calls that fn(*args, **kw) would make (fn: a function of this module, or any
    function built from them) without making them."""
    global _recording
    assert _recording is None, "prepare() does not nest"
    rec = Prepared()
    _recording = rec
    try:
        fn(*args, **kw)
    finally:
        _recording = None
    return rec


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return ctypes.c_void_p(t.data_ptr())


def _ptr_addressable(t: torch.Tensor):
    """Device tensor, or a CPU tensor in pinned memory (which the GPU addresses at the same pointer)."""
    assert t.is_contiguous() and (t.is_cuda or t.is_pinned()), "need a CUDA tensor or a pinned CPU tensor"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def make_problem(B, Hq, Hkv, d, S, dtype, max_blocks, k, ctx_len: torch.Tensor, sm_scale: float = 0.0,
                 n_sink: int = 0, n_tail: int = 0, group_max: int = 0, per_head: int = 0,
                 digest_kind: int = 0, tile_stride: int = 0):
    assert ctx_len.dtype == torch.int32 and ctx_len.is_cuda
    return Problem(B, Hq, Hkv, d, S, dtype, max_blocks, k, float(sm_scale), int(n_sink), int(n_tail),
                   int(group_max), int(per_head), int(digest_kind), int(tile_stride), ctx_len.data_ptr())


def version() -> int:
    return lib().scout_version()


def set_attn_mode(family: int = 0, nsplit: int = 0, waves: int = 0):
    _check("scout_set_attn_mode", lib().scout_set_attn_mode(family, nsplit, waves))


def workspace_bytes(p: Problem) -> int:
    n = ctypes.c_size_t(0)
    _check("scout_workspace_bytes", lib().scout_workspace_bytes(ctypes.byref(p), ctypes.byref(n)))
    return n.value


def alloc_workspace(p: Problem, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(p), dtype=torch.uint8, device=device)


def calib_copy(src: torch.Tensor, dst: torch.Tensor):
    n = src.numel() * src.element_size()
    _call("scout_calib_copy", calib_lib().scout_calib_copy, _ptr(src), _ptr(dst), n, _stream())


def build_digests(p: Problem, k_blocks, digest):
    _call("build_digests", lib().build_digests, ctypes.byref(p), _ptr(k_blocks), _ptr(digest), _stream())


def append_token(p: Problem, ctx_len, k_new, v_new, new_slot, digest, block_table, k_pool, v_pool, n_slots,
                 host_k=None, host_v=None):
    """host_k / host_v: the host's copy of every block (pinned CPU tensors, or device tensors), or None."""
    hk = None if host_k is None else _ptr_addressable(host_k)
    hv = None if host_v is None else _ptr_addressable(host_v)
    _call("append_token", lib().append_token, ctypes.byref(p), _ptr(ctx_len), _ptr(k_new), _ptr(v_new),
          _ptr(new_slot), _ptr(digest), _ptr(block_table), _ptr(k_pool),
          _ptr(v_pool), int(n_slots), hk, hv, _stream())


def score_blocks(p: Problem, q, digest, scores, ws):
    _call("score_blocks", lib().score_blocks, ctypes.byref(p), _ptr(q), _ptr(digest), _ptr(scores),
          _ptr(ws), ws.numel(), _stream())


def select_topk(p: Problem, scores, block_table, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, ws):
    _call("select_topk", lib().select_topk, ctypes.byref(p), _ptr(scores), _ptr(block_table), _ptr(sel_all),
          _ptr(sel_gpu), _ptr(slot_gpu), _ptr(n_gpu), _ptr(sel_host),
          _ptr(n_host), _ptr(ws), ws.numel(), _stream())


def sparse_decode_attn(p: Problem, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, o, m, l, ws):
    _call("sparse_decode_attn", lib().sparse_decode_attn, ctypes.byref(p), _ptr(q), _ptr(k_pool), _ptr(v_pool), int(n_slots),
          _ptr(sel_gpu), _ptr(slot_gpu), _ptr(n_gpu), _ptr(o), _ptr(m), _ptr(l),
          _ptr(ws), ws.numel(), _stream())


def sparse_decode_attn_static(p: Problem, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, o, m, l):
    """sparse_decode_attn without a workspace: the library's own static scratch buffer (no allocation)."""
    _call("sparse_decode_attn_static", lib().sparse_decode_attn_static, ctypes.byref(p), _ptr(q), _ptr(k_pool),
          _ptr(v_pool), int(n_slots), _ptr(sel_gpu), _ptr(slot_gpu), _ptr(n_gpu), _ptr(o), _ptr(m), _ptr(l), _stream())


def attn_partials(p: Problem, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, ws):
    _call("scout_attn_partials", lib().scout_attn_partials, ctypes.byref(p), _ptr(q), _ptr(k_pool), _ptr(v_pool), int(n_slots),
          _ptr(sel_gpu), _ptr(slot_gpu), _ptr(n_gpu), _ptr(ws), ws.numel(),
          _stream())


def attn_finish(p: Problem, host_o, host_m, host_l, out, lse, ws):
    _call("scout_attn_finish", lib().scout_attn_finish, ctypes.byref(p), _ptr(host_o), _ptr(host_m), _ptr(host_l),
          _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream())


def merge_partials(p: Problem, o_a, m_a, l_a, o_b, m_b, l_b, out, lse=None):
    _call("merge_partials", lib().merge_partials, ctypes.byref(p), _ptr(o_a), _ptr(m_a), _ptr(l_a), _ptr(o_b),
          _ptr(m_b), _ptr(l_b), _ptr(out), _ptr(lse), _stream())


def periodic_recall(p: Problem, q, digest, block_table, recall_blk, recall_slot, evict_blk, n_recall, ws):
    _call("periodic_recall", lib().periodic_recall, ctypes.byref(p), _ptr(q), _ptr(digest), _ptr(block_table), _ptr(recall_blk),
          _ptr(recall_slot), _ptr(evict_blk), _ptr(n_recall), _ptr(ws), ws.numel(),
          _stream())


def recall_fetch(p: Problem, src_k, src_v, recall_blk, recall_slot, n_recall, k_pool, v_pool, n_slots):
    """src_k / src_v: tensors in pinned host memory or on the device."""
    _call("recall_fetch", lib().recall_fetch, ctypes.byref(p), _ptr_addressable(src_k), _ptr_addressable(src_v), _ptr(recall_blk),
          _ptr(recall_slot), _ptr(n_recall), _ptr(k_pool), _ptr(v_pool),
          int(n_slots), _stream())


def recall_scatter(p: Problem, staged, tile_off, recall_blk, recall_slot, n_recall, k_pool, v_pool, n_slots):
    """staged: device buffer of packed tiles [tiles][2][S][d]; tile_off: first tile of each pair."""
    tile_elems = p.S * p.d * 2
    assert staged.numel() % tile_elems == 0
    _call("recall_scatter", lib().recall_scatter, ctypes.byref(p), _ptr(staged), staged.numel() // tile_elems,
          _ptr(tile_off), _ptr(recall_blk),
          _ptr(recall_slot), _ptr(n_recall), _ptr(k_pool), _ptr(v_pool), int(n_slots), _stream())


def calib_read(src, nbytes: int, sink=None):
    _call("scout_calib_read", calib_lib().scout_calib_read, _ptr(src), int(nbytes), _ptr(sink), _stream())


def calib_gather(p: Problem, k_pool, v_pool, n_slots, slot_gpu, n_gpu, sink=None):
    _call("scout_calib_gather", calib_lib().scout_calib_gather, ctypes.byref(p), _ptr(k_pool), _ptr(v_pool), int(n_slots),
          _ptr(slot_gpu), _ptr(n_gpu), _ptr(sink), _stream())


def layer_step(p: Problem, q, digest, block_table, k_pool, v_pool, n_slots, host_o, host_m, host_l, scores,
               sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, out, lse, ws):
    _call("scout_layer_step", lib().scout_layer_step, ctypes.byref(p), _ptr(q), _ptr(digest), _ptr(block_table), _ptr(k_pool),
          _ptr(v_pool), int(n_slots), _ptr(host_o), _ptr(host_m), _ptr(host_l),
          _ptr(scores), _ptr(sel_all), _ptr(sel_gpu), _ptr(slot_gpu), _ptr(n_gpu),
          _ptr(sel_host), _ptr(n_host), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
          _stream())
