"""CPU-side checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and rejects malformed arguments on the host before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2506_19225_amd import vxl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(headers=("vxl.h", "vxl_debug.h")):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(vxl_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def exported_symbols():
    """Dynamic symbols of libvxl.so whose names start with vxl_ (the C ABI; C++ names are mangled)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", vxl.LIB_PATH], capture_output=True, text=True, check=True)
    return sorted({ln.split()[-1] for ln in out.stdout.splitlines() if ln.split() and ln.split()[-1].startswith("vxl_")})


def test_library_exports_every_declared_symbol():
    lib = vxl.lib()
    names = declared_symbols()
    assert {"vxl_chunk_prefill", "vxl_chunk_score_topk", "vxl_gather_bilevel_kv", "vxl_bilevel_decode",
            "vxl_layout_create", "vxl_layout_destroy", "vxl_workspace_bytes", "vxl_mixed_kv_capacity",
            "vxl_status_string", "vxl_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libvxl.so does not export {n}"
    assert lib.vxl_version() >= 100
    assert lib.vxl_status_string(0) == b"ok"
    assert b"workspace" in lib.vxl_status_string(vxl.VXL_ERR_WORKSPACE)
    assert b"allocat" in lib.vxl_status_string(vxl.VXL_ERR_ALLOC)


def test_library_exports_nothing_that_no_header_declares():
    undeclared = set(exported_symbols()) - set(declared_symbols())
    assert not undeclared, f"exported but declared in no header under include/: {sorted(undeclared)}"
    debug = set(declared_symbols(("vxl_debug.h",)))
    assert debug and all(n.startswith("vxl_debug_") for n in debug)
    assert not any(n.startswith("vxl_debug_") for n in declared_symbols(("vxl.h",)))


def test_headers_are_plain_c_and_the_library_links_from_c(tmp_path):
    """The boundary is a C ABI: both headers compile as strict C99 (no C++ types, no torch), and a C
    program that links libvxl.so can call it without Python."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_vxl.c"
    src.write_text(
        '#include <stdio.h>\n#include "vxl.h"\n#include "vxl_debug.h"\n'
        'int main(void) {\n'
        '    int32_t bounds[3] = {2, 6, 9}, soff[3] = {0, 1, 2}, sidx[2] = {2, 6};\n'
        '    vxl_layout* h = NULL;\n'
        '    vxl_status st = vxl_layout_create(10, 2, 2, bounds, soff, sidx, NULL, &h);   /* last bound != n_tokens */\n'
        '    printf("%d %d %s|%d\\n", vxl_version(), (int)st, vxl_status_string(st), h == NULL);\n'
        '    return 0;\n}\n')
    exe = tmp_path / "use_vxl"
    libdir = os.path.dirname(vxl.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-l:libvxl.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout
    version, status, rest = out.split(" ", 2)
    assert int(version) >= 100 and int(status) == vxl.VXL_ERR_INVALID_ARG and rest.strip().endswith("|1")


def test_failing_runtime_call_is_reported_as_hip_error():
    """Without a GPU the first runtime call of vxl_layout_create (well-formed arguments) fails: the
    call must return VXL_ERR_HIP, leave the handle null and keep the text of the failing call."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible: no runtime call fails here")
    st, h = create(10, 2, [2, 6, 10], [0, 1, 2], [2, 6])
    assert st == vxl.VXL_ERR_HIP and not h.value
    assert len(vxl.lib().vxl_last_error()) > 0
    assert b"HIP" in vxl.lib().vxl_status_string(st)


def create(n_tokens, n_prefix, bounds, soff, sidx):
    b = np.asarray(bounds, np.int32)
    o = np.asarray(soff, np.int32)
    i = np.asarray(sidx, np.int32)
    h = C.c_void_p()
    st = vxl.lib().vxl_layout_create(n_tokens, n_prefix, len(b) - 1, b.ctypes.data, o.ctypes.data,
                                     i.ctypes.data if i.size else None, None, C.byref(h))
    return st, h


@pytest.mark.parametrize("args", [
    (10, 2, [2, 6, 9], [0, 1, 2], [2, 6]),          # last bound != n_tokens
    (10, 2, [3, 6, 10], [0, 1, 2], [3, 6]),         # first bound != n_prefix
    (10, 2, [2, 6, 6, 10], [0, 1, 1, 2], [2, 6]),   # empty chunk
    (10, 2, [2, 6, 10], [1, 1, 2], [2, 6]),         # offsets do not start at 0
    (10, 2, [2, 6, 10], [0, 2, 1], [2, 3]),         # offsets decrease
    (10, 2, [2, 6, 10], [0, 1, 2], [6, 7]),         # kept id outside its chunk
    (10, 2, [2, 6, 10], [0, 2, 3], [3, 3, 7]),      # duplicate kept id
    (10, 2, [2, 6, 10], [0, 2, 3], [4, 3, 7]),      # unsorted kept ids
    (0, 0, [0], [0], []),                           # no tokens
])
def test_layout_create_rejects_malformed_layouts_on_the_host(args):
    st, h = create(*args)
    assert st == vxl.VXL_ERR_INVALID_ARG and not h.value


def test_layout_create_rejects_null_and_oversized():
    h = C.c_void_p()
    assert vxl.lib().vxl_layout_create(4, 0, 1, None, None, None, None, C.byref(h)) == vxl.VXL_ERR_INVALID_ARG
    n = vxl.MAX_CHUNKS + 1
    st, h = create(n, 0, list(range(n + 1)), [0] * (n + 1), [])
    assert st == vxl.VXL_ERR_UNSUPPORTED


def test_windowed_layout_rejects_negative_window():
    b = np.asarray([2, 6, 10], np.int32)
    o = np.asarray([0, 1, 2], np.int32)
    i = np.asarray([2, 6], np.int32)
    h = C.c_void_p()
    st = vxl.lib().vxl_layout_create_windowed(10, 2, 2, b.ctypes.data, o.ctypes.data, i.ctypes.data, -1, None,
                                              C.byref(h))
    assert st == vxl.VXL_ERR_INVALID_ARG and not h.value


def test_hot_calls_reject_bad_descriptors_before_launch():
    lib = vxl.lib()
    fake = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    for desc, want in [
        (vxl.make_desc(28, 4, 96, "bf16"), vxl.VXL_ERR_UNSUPPORTED),
        (vxl.make_desc(28, 5, 128, "bf16"), vxl.VXL_ERR_INVALID_ARG),
        (vxl.make_desc(28, 4, 128, "bf16", -1.0), vxl.VXL_ERR_INVALID_ARG),
        (vxl.AttnDesc(28, 4, 128, 7, 0.0), vxl.VXL_ERR_UNSUPPORTED),
    ]:
        st = lib.vxl_bilevel_decode(C.byref(desc), fake, 1, 1, fake, fake, 64, fake, fake, None, fake, 1 << 20, None)
        assert st == want
        assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(desc), 1, 1, 64) == 0
    good = vxl.make_desc(28, 4, 128, "bf16")
    assert lib.vxl_bilevel_decode(C.byref(good), None, 1, 1, fake, fake, 64, fake, fake, None, fake, 1 << 20, None) \
        == vxl.VXL_ERR_INVALID_ARG
    assert lib.vxl_bilevel_decode(C.byref(good), fake, 0, 1, fake, fake, 64, fake, fake, None, fake, 1 << 20, None) \
        == vxl.VXL_ERR_INVALID_ARG
    odd = C.c_void_p(0x1004)           # misaligned base pointer
    assert lib.vxl_bilevel_decode(C.byref(good), odd, 1, 1, fake, fake, 64, fake, fake, None, fake, 1 << 20, None) \
        == vxl.VXL_ERR_INVALID_ARG
    assert lib.vxl_bilevel_decode(C.byref(good), fake, 1, 1, fake, fake, 4096, fake, fake, None, None, 0, None) \
        == vxl.VXL_ERR_WORKSPACE
    assert lib.vxl_chunk_prefill(None, C.byref(good), fake, fake, fake, fake, None, fake, 1 << 20, None) \
        == vxl.VXL_ERR_INVALID_ARG
    assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(good), 1, 32, 4096) > 0
    assert lib.vxl_mixed_kv_capacity(None, 3) == 0


def test_descriptor_strides_are_checked_on_the_host():
    """All four strides or none; positive multiples of 16 bytes; a token stride that holds a row."""
    lib = vxl.lib()
    fake = C.c_void_p(0x1000)
    ok = vxl.make_desc(28, 4, 128, "bf16", token_major=True)
    assert (ok.q_stride_head, ok.q_stride_tok, ok.kv_stride_head, ok.kv_stride_tok) == (128, 28 * 128, 128, 4 * 128)
    assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(ok), 1, 1, 64) > 0
    for bad in ((128, 0, 128, 512), (128, 3584, 128, 64), (128, 3588, 128, 512), (-8, 3584, 128, 512),
                (0, 3584, 0, 512)):
        d = vxl.make_desc(28, 4, 128, "bf16")
        d.q_stride_head, d.q_stride_tok, d.kv_stride_head, d.kv_stride_tok = bad
        assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(d), 1, 1, 64) == 0, bad
        st = lib.vxl_bilevel_decode(C.byref(d), fake, 1, 1, fake, fake, 64, fake, fake, None, fake, 1 << 20, None)
        assert st == vxl.VXL_ERR_INVALID_ARG, bad
    f32 = vxl.make_desc(4, 2, 64, "f32")
    f32.q_stride_head, f32.q_stride_tok, f32.kv_stride_head, f32.kv_stride_tok = (64, 260, 64, 132)   # multiples of 4
    assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(f32), 1, 1, 64) > 0
    r = vxl.make_desc(28, 4, 128, "bf16")
    r.reserved = 1
    assert lib.vxl_workspace_bytes(vxl.OP_DECODE, None, C.byref(r), 1, 1, 64) == 0
