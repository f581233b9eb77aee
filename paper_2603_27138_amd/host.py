"""ctypes binding of the host-side worker (include/scout_host.h): argument marshalling only.

The arrays are numpy arrays or CPU torch tensors; the worker keeps their pointers from submit to
wait, so the wrapper holds references until then.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# SCOUT_HOST_LIB names another build of the same source (the tests' sanitizer build) to load instead
LIB_PATH = os.environ.get("SCOUT_HOST_LIB") or os.path.join(HERE, "libscout_host.so")
EXPORTS = ["scout_host_create", "scout_host_destroy", "scout_host_submit", "scout_host_stage_recall", "scout_host_wait",
           "scout_host_done"]
F32, BF16 = 0, 1


class HostProblem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("S", ctypes.c_int32), ("dtype", ctypes.c_int32), ("max_blocks", ctypes.c_int32),
                ("k", ctypes.c_int32), ("sm_scale", ctypes.c_float)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2603_27138_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.scout_host_create.argtypes = [ctypes.c_int, ctypes.POINTER(vp)]
        L.scout_host_destroy.argtypes = [vp]
        L.scout_host_destroy.restype = None
        L.scout_host_submit.argtypes = [vp, ctypes.POINTER(HostProblem)] + [vp] * 9
        L.scout_host_stage_recall.argtypes = [vp, ctypes.POINTER(HostProblem)] + [vp] * 5 + [ctypes.c_size_t, vp,
                                                                                       ctypes.POINTER(ctypes.c_int64)]
        L.scout_host_wait.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
        L.scout_host_done.argtypes = [vp]
        _lib = L
    return _lib


def _addr(a):
    if isinstance(a, np.ndarray):
        assert a.flags["C_CONTIGUOUS"]
        return ctypes.c_void_p(a.ctypes.data)
    assert not a.is_cuda and a.is_contiguous(), "host worker takes CPU tensors"
    return ctypes.c_void_p(a.data_ptr())


class HostWorker:
    """A pool of worker threads computing the host's partial attention (Alg. 1 CPUAttn)."""

    def __init__(self, n_threads: int):
        self._h = ctypes.c_void_p()
        rc = lib().scout_host_create(int(n_threads), ctypes.byref(self._h))
        if rc != 0:
            raise RuntimeError(f"scout_host_create failed ({rc})")
        self._keep = []      # the arrays of the jobs handed in and not yet waited for

    def submit(self, p: HostProblem, q, k_blocks, v_blocks, sel_host, n_host, ctx_len, o, m, l):
        args = (q, k_blocks, v_blocks, sel_host, n_host, ctx_len, o, m, l)
        rc = lib().scout_host_submit(self._h, ctypes.byref(p), *[_addr(a) for a in args])
        if rc != 0:
            raise RuntimeError(f"scout_host_submit failed ({rc})")
        if p.B * p.Hkv > 0:
            self._keep.append((p,) + args)

    def stage_recall(self, p: HostProblem, k_blocks, v_blocks, recall_blk, n_recall, staged, tile_off) -> int:
        """Starts packing the tiles a recall plan names into `staged` (Sec. 3.4); tile_off is filled before
        this returns.  Returns the number of tiles; wait() as after submit."""
        total = ctypes.c_int64(0)
        nbytes = staged.nbytes if isinstance(staged, np.ndarray) else staged.numel() * staged.element_size()
        rc = lib().scout_host_stage_recall(self._h, ctypes.byref(p), _addr(k_blocks), _addr(v_blocks),
                                           _addr(recall_blk), _addr(n_recall), _addr(staged), nbytes,
                                           _addr(tile_off), ctypes.byref(total))
        if rc != 0:
            raise RuntimeError(f"scout_host_stage_recall failed ({rc})")
        if total.value:
            self._keep.append((p, k_blocks, v_blocks, recall_blk, n_recall, staged, tile_off))
        return total.value

    def wait(self) -> float:
        """Blocks until the oldest job not yet waited for is done (up to two may be outstanding: one
        running, one behind it); returns the seconds it ran."""
        sec = ctypes.c_double(0.0)
        rc = lib().scout_host_wait(self._h, ctypes.byref(sec))
        if rc != 0:
            raise RuntimeError(f"scout_host_wait failed ({rc})")
        if self._keep:
            self._keep.pop(0)
        return sec.value

    def done(self) -> bool:
        return bool(lib().scout_host_done(self._h))

    def close(self):
        if self._h:
            lib().scout_host_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
