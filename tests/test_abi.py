"""The C-ABI library loads, exports every declared symbol and rejects bad arguments on the host.

Runs without a GPU: every call here must fail validation before anything is launched
(pointers are fake, never dereferenced).
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2603_27138_amd import build
    if not os.path.exists(build.LIB):
        build.build()
    from paper_2603_27138_amd import binding
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "scout.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    syms = declared_symbols()
    assert {"score_blocks", "select_topk", "sparse_decode_attn", "merge_partials", "periodic_recall"} <= set(syms)
    L = lib.lib()
    for s in syms:
        assert hasattr(L, s), s
    assert sorted(lib.EXPORTS) == syms
    assert L.scout_version() >= 100
    assert L.scout_strerror(-1) == b"invalid argument"


def test_calibration_library_is_separate_and_exports_its_header(lib):
    """The measurement aids are not in the product library: libscout.so exports none of them, and
    libscout_calib.so exports what include/scout_calib.h declares."""
    text = open(os.path.join(ROOT, "include", "scout_calib.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    syms = sorted(set(re.findall(r"\bint\s+(scout_calib_\w+)\s*\(", text)))
    assert syms == sorted(lib.CALIB_EXPORTS) and len(syms) == 3
    for s_ in syms:
        assert hasattr(lib.calib_lib(), s_), s_
        assert not hasattr(lib.lib(), s_), s_
    assert lib.calib_lib().scout_calib_copy(None, None, 16, None) == lib.EINVAL
    assert lib.calib_lib().scout_calib_read(FAKE, 24, None, None) == lib.EINVAL
    assert lib.calib_lib().scout_calib_gather(None, FAKE, FAKE, 4, FAKE, FAKE, None, None) == lib.EINVAL


def test_host_library_exports_every_declared_symbol():
    from paper_2603_27138_amd import build, host
    if not os.path.exists(build.HOST_LIB):
        build.build_host()
    text = open(os.path.join(ROOT, "include", "scout_host.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    syms = sorted(set(re.findall(r"\b(?:int|void)\s+(scout_host_\w+)\s*\(", text)))
    assert len(syms) == 6 and sorted(host.EXPORTS) == syms
    for s_ in syms:
        assert hasattr(host.lib(), s_), s_


def _problem(lib, **kw):
    base = dict(B=2, Hq=8, Hkv=2, d=128, S=32, dtype=lib.BF16, max_blocks=64, k=8, sm_scale=0.0, ctx_len=0x1000)
    base.update(kw)
    return lib.Problem(**base)


FAKE = ctypes.c_void_p(0x10000)   # 16-byte aligned, never dereferenced


def test_workspace_bytes(lib):
    n = ctypes.c_size_t(0)
    assert lib.lib().scout_workspace_bytes(ctypes.byref(_problem(lib)), ctypes.byref(n)) == 0
    assert n.value > 0 and n.value % 256 == 0
    assert lib.lib().scout_workspace_bytes(None, ctypes.byref(n)) == lib.EINVAL
    assert lib.lib().scout_workspace_bytes(ctypes.byref(_problem(lib)), None) == lib.EINVAL


@pytest.mark.parametrize("kw,code", [
    (dict(Hq=7), -1), (dict(Hkv=0), -1), (dict(B=-1), -1), (dict(k=0), -1), (dict(max_blocks=0), -1),
    (dict(dtype=5), -1), (dict(sm_scale=-1.0), -1), (dict(ctx_len=None), -1), (dict(n_sink=-1), -1), (dict(n_tail=-3), -1), (dict(group_max=2), -1), (dict(per_head=2), -1), (dict(digest_kind=2), -1), (dict(digest_kind=1, group_max=1), -2), (dict(per_head=-1), -1), (dict(tile_stride=100), -1), (dict(tile_stride=4100), -1), (dict(tile_stride=-8192), -1), (dict(B=70000), -2),
    (dict(d=96), -2), (dict(S=8), -2), (dict(Hq=64, Hkv=2), -2), (dict(k=5000), -2), (dict(max_blocks=1 << 20), -2),
])
def test_bad_problem_is_rejected_before_launch(lib, kw, code):
    p = _problem(lib, **kw)
    L = lib.lib()
    assert L.score_blocks(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == code
    assert L.merge_partials(ctypes.byref(p), FAKE, FAKE, FAKE, None, None, None, FAKE, None, None) == code
    assert L.build_digests(ctypes.byref(p), FAKE, FAKE, None) == code


def test_null_misaligned_and_workspace_errors(lib):
    p = _problem(lib)
    L = lib.lib()
    odd = ctypes.c_void_p(0x10004)
    assert L.score_blocks(ctypes.byref(p), None, FAKE, FAKE, FAKE, 1 << 30, None) == lib.EINVAL
    assert L.score_blocks(ctypes.byref(p), odd, FAKE, FAKE, FAKE, 1 << 30, None) == lib.EINVAL
    assert L.select_topk(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 30, None) == lib.EINVAL
    args = [FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE]
    assert L.sparse_decode_attn(ctypes.byref(p), *args, None, 0, None) == lib.EWORKSPACE
    assert L.sparse_decode_attn(ctypes.byref(p), *args, FAKE, 16, None) == lib.EWORKSPACE
    assert L.sparse_decode_attn(ctypes.byref(p), *args, ctypes.c_void_p(0x10010), 1 << 30, None) == lib.EWORKSPACE
    args[3] = -1
    assert L.sparse_decode_attn(ctypes.byref(p), *args, FAKE, 1 << 30, None) == lib.EINVAL
    # host partial must be given completely or not at all
    assert L.merge_partials(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, None) == lib.EINVAL
    assert L.periodic_recall(ctypes.byref(p), FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == lib.EINVAL
    assert L.recall_scatter(ctypes.byref(p), None, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, None) == lib.EINVAL
    assert L.recall_scatter(ctypes.byref(p), odd, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, None) == lib.EINVAL
    assert L.recall_scatter(ctypes.byref(p), FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, -1, None) == lib.EINVAL
    assert L.recall_scatter(ctypes.byref(p), FAKE, -4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, None) == lib.EINVAL
    assert L.recall_fetch(ctypes.byref(p), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 4, None) == lib.EINVAL
    assert L.scout_set_attn_mode(5, 0, 0) == lib.EINVAL and L.scout_set_attn_mode(0, 0, 5) == lib.EINVAL and L.scout_set_attn_mode(0, 0, 0) == 0
    # MFMA family forced on a shape it does not cover
    p32 = _problem(lib, dtype=lib.F32)
    assert L.scout_set_attn_mode(2, 0, 0) == 0
    try:
        args[3] = 10
        assert L.sparse_decode_attn(ctypes.byref(p32), *args, FAKE, 1 << 30, None) == lib.EUNSUPPORTED
    finally:
        L.scout_set_attn_mode(0, 0, 0)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_27138_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "scout_oracle" not in text, f


def test_static_scratch_entry_point_rejects_on_the_host(lib):
    """sparse_decode_attn_static validates like sparse_decode_attn, and a problem whose per-split partials
    exceed the static buffer gets SCOUT_ESCRATCH before anything is looked up or launched."""
    L = lib.lib()
    p = _problem(lib)
    args = [FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE]
    assert L.sparse_decode_attn_static(ctypes.byref(p), None, *args[1:], None) == lib.EINVAL
    assert L.sparse_decode_attn_static(ctypes.byref(p), ctypes.c_void_p(0x10004), *args[1:], None) == lib.EINVAL
    bad = list(args)
    bad[3] = -1
    assert L.sparse_decode_attn_static(ctypes.byref(p), *bad, None) == lib.EINVAL
    assert L.sparse_decode_attn_static(ctypes.byref(_problem(lib, d=96)), *args, None) == lib.EUNSUPPORTED
    # fp32, 512 pairs of 16 heads: two splits per pair make 16384 rows of 128 floats = 8 MiB of o alone
    big = _problem(lib, B=64, Hq=128, Hkv=8, dtype=lib.F32)
    assert L.sparse_decode_attn_static(ctypes.byref(big), *args, None) == lib.ESCRATCH
    assert b"static" in L.scout_strerror(lib.ESCRATCH)
    assert lib.STATIC_SCRATCH_BYTES == 8 << 20
    text = open(os.path.join(ROOT, "include", "scout.h")).read()
    assert "#define SCOUT_STATIC_SCRATCH_BYTES (8u << 20)" in text


def test_attention_mode_belongs_to_the_calling_thread(lib):
    """scout_set_attn_mode in one thread leaves every other thread's setting alone (observable without a
    GPU: the fp32 problem that is too large for the static scratch is refused as unsupported where the
    MFMA family is forced, and for its size where the choice is automatic)."""
    import threading
    L = lib.lib()
    big = _problem(lib, B=64, Hq=128, Hkv=8, dtype=lib.F32)
    args = [FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE]
    seen = {}

    def other():
        assert L.scout_set_attn_mode(2, 0, 0) == 0
        seen["forced"] = L.sparse_decode_attn_static(ctypes.byref(big), *args, None)

    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert seen["forced"] == lib.EUNSUPPORTED
    assert L.sparse_decode_attn_static(ctypes.byref(big), *args, None) == lib.ESCRATCH


def test_headers_are_plain_c_and_the_binding_has_the_header_layout(lib, tmp_path):
    """The three headers compile as C99 with no warnings, a C program links against the library and
    calls its host-only entry points, and the struct the Python binding marshals has the size and the
    field offsets of the header's."""
    import subprocess
    from paper_2603_27138_amd import build
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "scout.h"
#include "scout_calib.h"
#include "scout_host.h"
int main(void) {
  scout_problem p = {0};
  size_t bytes = 0;
  int rc;
  p.B = 2; p.Hq = 8; p.Hkv = 2; p.d = 128; p.S = 32; p.dtype = SCOUT_BF16; p.max_blocks = 100; p.k = 8;
  printf("%d\n", scout_version());
  printf("%s\n", scout_strerror(SCOUT_EWORKSPACE));
  rc = scout_workspace_bytes(&p, &bytes);
  printf("%d %zu\n", rc, bytes);
  p.d = 96;
  rc = scout_workspace_bytes(&p, &bytes);
  printf("%d\n", rc);
  printf("%zu", sizeof(scout_problem));
  printf(" %zu %zu %zu %zu %zu\n", offsetof(scout_problem, B), offsetof(scout_problem, sm_scale),
         offsetof(scout_problem, per_head), offsetof(scout_problem, tile_stride), offsetof(scout_problem, ctx_len));
  return 0;
}
''')
    exe = tmp_path / "abi"
    libdir = os.path.dirname(build.LIB)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
           "-o", str(exe), "-L", libdir, "-lscout", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
           "-Wl,--allow-shlib-undefined"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr
    lines = out.stdout.split("\n")
    assert int(lines[0]) == lib.lib().scout_version()
    assert lines[1] == lib.lib().scout_strerror(lib.EWORKSPACE).decode()
    rc, nbytes = lines[2].split()
    assert int(rc) == 0 and int(nbytes) > 0 and int(nbytes) % 256 == 0
    assert int(lines[3]) == lib.EUNSUPPORTED
    P = lib.Problem
    want = [ctypes.sizeof(P), P.B.offset, P.sm_scale.offset, P.per_head.offset, P.tile_stride.offset, P.ctx_len.offset]
    assert [int(x) for x in lines[4].split()] == want
