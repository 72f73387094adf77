"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/wgrad.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_1908_05460_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)      # non-null, 256-aligned, never dereferenced by validation


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return B.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "wgrad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv_wgrad_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS) and len(names) == 19
    for n in names:
        assert getattr(lib, n) is not None


def test_descriptor_struct_matches_header():
    assert ctypes.sizeof(B.ConvDesc) == 12 * 4
    d = B.desc(2, 3, 8, 6, 5, R=3, S=2, stride=2, pad=1, stride_w=1, pad_w=0)
    assert (d.Ho, d.Wo) == (4, 5)


def test_invalid_arguments_are_rejected_before_any_launch(lib):
    good = B.desc(2, 3, 8, 8, 4)
    f = lib.conv_wgrad_exact
    assert f(None, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), None, FAKE, FAKE, FAKE, 1 << 30, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), FAKE, None, FAKE, FAKE, 1 << 30, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), FAKE, FAKE, None, FAKE, 1 << 30, None) == B.INVALID_ARG
    for field, val in (("N", 0), ("C", -1), ("K", 0), ("R", 0), ("stride_h", 0), ("pad_w", -1), ("dtype", 7)):
        bad = B.desc(2, 3, 8, 8, 4)
        setattr(bad, field, val)
        assert f(ctypes.byref(bad), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.INVALID_ARG, field
        assert lib.conv_wgrad_zero(ctypes.byref(bad), FAKE, None) == B.INVALID_ARG
        assert B.workspace_bytes(bad, B.EXACT) == 0
    empty = B.desc(1, 1, 2, 2, 1, R=5, S=5, pad=1)          # filter larger than the padded input
    assert f(ctypes.byref(empty), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.INVALID_ARG
    assert lib.conv_wgrad_approx(ctypes.byref(good), FAKE, FAKE, None, 1.0, None, None, FAKE, 1 << 30, None) == B.INVALID_ARG
    assert lib.conv_wgrad_select(ctypes.byref(good), FAKE, None, FAKE, None) == B.INVALID_ARG
    assert lib.conv_wgrad_random(ctypes.byref(good), FAKE, -1.0, 0, 0, None) == B.INVALID_ARG
    assert lib.conv_wgrad_random(ctypes.byref(good), None, 1.0, 0, 0, None) == B.INVALID_ARG


def test_sizes_that_would_wrap_32_bit_arithmetic_are_refused(lib):
    """Output extents are computed in 64 bits: a huge padding on ONE axis must not wrap into a negative
    map length (with both axes huge the product of two negatives happened to look positive)."""
    for kw in (dict(pad=1 << 30, pad_w=1), dict(pad=1, pad_w=1 << 30), dict(pad=1 << 30, pad_w=1 << 30),
               dict(pad=(1 << 30) - 1, pad_w=0), dict(pad=40000, pad_w=1), dict(pad=1, pad_w=1, stride=40000)):
        d = B.desc(2, 3, 8, 8, 4, **kw)
        for method in (B.EXACT, B.APPROX):
            assert B.workspace_bytes(d, method) == 0, kw
        assert lib.conv_wgrad_zero(ctypes.byref(d), FAKE, None) == B.UNSUPPORTED, kw
        assert lib.conv_wgrad_approx(ctypes.byref(d), FAKE, FAKE, FAKE, 1.0, None, None, FAKE, 1 << 30, None) == B.UNSUPPORTED, kw
        assert lib.conv_wgrad_select(ctypes.byref(d), FAKE, FAKE, FAKE, None) == B.UNSUPPORTED, kw
        assert lib.conv_wgrad_approx_topk(ctypes.byref(d), FAKE, FAKE, FAKE, 2, 1.0, None, None, FAKE, 1 << 30, None) == B.UNSUPPORTED, kw
        assert lib.conv_wgrad_exact(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == B.UNSUPPORTED, kw
    # a map of 32767 rows is the largest a packed (row, col) holds; one more is refused
    ok = B.desc(1, 1, 32767, 4, 1, R=1, S=1, pad=0)
    assert lib.conv_wgrad_zero(ctypes.byref(ok), None, None) == B.INVALID_ARG        # geometry accepted, null dW
    too = B.desc(1, 1, 32768, 4, 1, R=1, S=1, pad=0)
    assert lib.conv_wgrad_zero(ctypes.byref(too), FAKE, None) == B.UNSUPPORTED


def test_static_scratch_call_validates_and_enforces_its_limit_on_the_host(lib):
    """conv_wgrad_approx_static: arguments and the size limit are checked before the GPU is touched."""
    f = lib.conv_wgrad_approx_static
    good = B.desc(16, 16, 32, 32, 16)
    assert B.workspace_bytes(good, B.APPROX) <= B.STATIC_SCRATCH_BYTES
    assert f(None, FAKE, FAKE, FAKE, 1.0, None, None, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), None, FAKE, FAKE, 1.0, None, None, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), FAKE, None, FAKE, 1.0, None, None, None) == B.INVALID_ARG
    assert f(ctypes.byref(good), FAKE, FAKE, None, 1.0, None, None, None) == B.INVALID_ARG
    big = B.desc(2048, 512, 4, 4, 512)              # batch 2048 of a 512 -> 512 layer: partial sums beyond 24 MiB
    assert B.workspace_bytes(big, B.APPROX) > B.STATIC_SCRATCH_BYTES
    assert f(ctypes.byref(big), FAKE, FAKE, FAKE, 1.0, None, None, None) == B.SCRATCH_LIMIT
    header = open(os.path.join(ROOT, "include", "wgrad.h")).read()
    assert "#define WGRAD_STATIC_SCRATCH_BYTES (24u << 20)" in header and B.STATIC_SCRATCH_BYTES == 24 << 20
    assert b"static buffer" in lib.conv_wgrad_status_string(B.SCRATCH_LIMIT)


def test_workspace_is_checked(lib):
    d = B.desc(128, 16, 32, 32, 16)
    for method, call in ((B.EXACT, lambda ws, n: lib.conv_wgrad_exact(ctypes.byref(d), FAKE, FAKE, FAKE, ws, n, None)),
                         (B.APPROX, lambda ws, n: lib.conv_wgrad_approx(ctypes.byref(d), FAKE, FAKE, FAKE, 1.0, None, None, ws, n, None))):
        need = B.workspace_bytes(d, method)
        assert need > 0 and need % 256 == 0
        assert call(FAKE, need - 1) == B.WORKSPACE_TOO_SMALL
        assert call(None, need) == B.WORKSPACE_TOO_SMALL
        assert call(ctypes.c_void_p(0x1010), need) == B.WORKSPACE_TOO_SMALL      # misaligned
    assert B.workspace_bytes(d, B.ZERO) == 0 and B.workspace_bytes(d, B.RANDOM) == 0


def test_topk_limits_and_workspace_are_checked_on_the_host(lib):
    d = B.desc(16, 16, 32, 32, 16)
    f = lib.conv_wgrad_approx_topk
    for k in (0, -3, 65, 32 * 32 + 1):
        assert B.topk_workspace_bytes(d, k) == 0
        assert f(ctypes.byref(d), FAKE, FAKE, FAKE, k, 1.0, None, None, FAKE, 1 << 30, None) == B.UNSUPPORTED
    tiny = B.desc(4, 8, 2, 2, 8)
    assert B.topk_workspace_bytes(tiny, 4) > 0 and B.topk_workspace_bytes(tiny, 5) == 0
    need = B.topk_workspace_bytes(d, 8)
    assert need >= 16 * 16 * 8 * 4 and need % 256 == 0
    assert f(ctypes.byref(d), FAKE, FAKE, FAKE, 8, 1.0, None, None, FAKE, need - 1, None) == B.WORKSPACE_TOO_SMALL
    assert f(ctypes.byref(d), FAKE, FAKE, FAKE, 8, 1.0, None, None, None, need, None) == B.WORKSPACE_TOO_SMALL
    assert f(ctypes.byref(d), None, FAKE, FAKE, 8, 1.0, None, None, FAKE, need, None) == B.INVALID_ARG
    bad = B.desc(16, 16, 32, 32, 0)
    assert f(ctypes.byref(bad), FAKE, FAKE, FAKE, 1, 1.0, None, None, FAKE, need, None) == B.INVALID_ARG


def test_layout_calls_validate_on_the_host(lib):
    d = B.desc(16, 16, 32, 32, 16)
    for method in (B.EXACT, B.APPROX):
        need = B.nhwc_workspace_bytes(d, method)
        assert need > 0 and need % 256 == 0
    assert B.nhwc_workspace_bytes(d, B.EXACT) >= 16 * 16 * 32 * 32 * 4 + B.workspace_bytes(d, B.EXACT)
    assert B.nhwc_workspace_bytes(d, B.ZERO) == 0
    ap, ex = lib.conv_wgrad_approx_nhwc, lib.conv_wgrad_exact_nhwc
    need = B.nhwc_workspace_bytes(d, B.APPROX)
    assert ap(ctypes.byref(d), FAKE, FAKE, FAKE, 3, 1.0, None, None, FAKE, need, None) == B.INVALID_ARG     # layout
    assert ap(ctypes.byref(d), FAKE, FAKE, FAKE, -1, 1.0, None, None, FAKE, need, None) == B.INVALID_ARG
    assert ap(ctypes.byref(d), None, FAKE, FAKE, 1, 1.0, None, None, FAKE, need, None) == B.INVALID_ARG
    assert ap(ctypes.byref(d), FAKE, FAKE, FAKE, 1, 1.0, None, None, FAKE, need - 1, None) == B.WORKSPACE_TOO_SMALL
    need = B.nhwc_workspace_bytes(d, B.EXACT)
    assert ex(ctypes.byref(d), FAKE, FAKE, FAKE, 7, FAKE, need, None) == B.INVALID_ARG
    assert ex(ctypes.byref(d), FAKE, FAKE, FAKE, 2, FAKE, need - 1, None) == B.WORKSPACE_TOO_SMALL
    assert ex(ctypes.byref(d), FAKE, FAKE, FAKE, 2, None, need, None) == B.WORKSPACE_TOO_SMALL
    tx, pm = lib.conv_wgrad_transpose_x, lib.conv_wgrad_permute_dw
    assert tx(ctypes.byref(d), 1, None, FAKE, None) == B.INVALID_ARG
    assert tx(ctypes.byref(d), 1, FAKE, FAKE, None) == B.INVALID_ARG           # in place
    assert pm(ctypes.byref(d), 0, 3, FAKE, ctypes.c_void_p(0x2000), None) == B.INVALID_ARG
    assert pm(ctypes.byref(d), 0, 1, FAKE, FAKE, None) == B.INVALID_ARG        # in place
    bad = B.desc(16, 16, 32, 32, 0)
    assert tx(ctypes.byref(bad), 1, FAKE, ctypes.c_void_p(0x2000), None) == B.INVALID_ARG
    assert B.nhwc_workspace_bytes(bad, B.APPROX) == 0


def test_schedule_validates_all_layers_first(lib):
    n = 3
    descs = (B.ConvDesc * n)(B.desc(4, 8, 8, 8, 8), B.desc(64, 8, 8, 8, 8), B.desc(4, 8, 8, 8, 0))
    ptrs = (ctypes.c_void_p * n)(0x1000, 0x1000, 0x1000)
    meth = (ctypes.c_uint8 * n)(B.ZERO, B.ZERO, B.ZERO)
    run = lib.conv_wgrad_schedule_run
    assert run(descs, ptrs, ptrs, ptrs, meth, n, 1.0, 1.0, 0, 0, FAKE, 1 << 30, None) == B.INVALID_ARG  # layer 3 bad
    descs[2].K = 8
    meth[1] = 9
    assert run(descs, ptrs, ptrs, ptrs, meth, n, 1.0, 1.0, 0, 0, FAKE, 1 << 30, None) == B.INVALID_ARG  # bad method
    meth[1] = B.EXACT
    assert B.workspace_bytes(descs[1], B.EXACT) > 0
    assert run(descs, ptrs, ptrs, ptrs, meth, n, 1.0, 1.0, 0, 0, FAKE, 0, None) == B.WORKSPACE_TOO_SMALL
    assert run(descs, ptrs, ptrs, ptrs, meth, 0, 1.0, 1.0, 0, 0, FAKE, 0, None) == B.INVALID_ARG
    assert lib.conv_wgrad_schedule_workspace_bytes(descs, meth, n) == B.workspace_bytes(descs[1], B.EXACT)


def test_status_strings(lib):
    seen = {B.status_string(s) for s in (0, -1, -2, -3, -4, -99)}
    assert len(seen) == 6 and B.status_string(0) == "ok"


C_CALLER = r"""
#include <stdio.h>
#include "wgrad.h"
int main(void)
{
    wgrad_conv_desc d = {128, 16, 32, 32, 16, 3, 3, 1, 1, 1, 1, WGRAD_F32};
    printf("%zu %zu %zu %zu\n", conv_wgrad_workspace_bytes(&d, WGRAD_EXACT), conv_wgrad_workspace_bytes(&d, WGRAD_APPROX),
           conv_wgrad_topk_workspace_bytes(&d, 4), conv_wgrad_nhwc_workspace_bytes(&d, WGRAD_APPROX));
    printf("%d %s\n", conv_wgrad_exact(&d, 0, 0, 0, 0, 0, 0), conv_wgrad_status_string(WGRAD_INVALID_ARG));
    return 0;
}
"""


def test_header_is_plain_c_and_a_c_program_can_call_the_library(lib, tmp_path):
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no gcc")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "caller.c"
    src.write_text(C_CALLER)
    # the header alone: strict C99 and C++
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run([gcc, "-x", "c++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    hip = "/opt/rocm/lib/libamdhip64.so"
    if not os.path.exists(hip):
        pytest.skip("no HIP runtime to link a C program against")
    exe = tmp_path / "caller"
    pkg = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", pkg, "-l:libwgrad.so", hip,
                    "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120).stdout.split("\n")
    d = B.desc(128, 16, 32, 32, 16)
    want = [B.workspace_bytes(d, B.EXACT), B.workspace_bytes(d, B.APPROX), B.topk_workspace_bytes(d, 4),
            B.nhwc_workspace_bytes(d, B.APPROX)]
    assert [int(x) for x in out[0].split()] == want
    assert out[1].split()[0] == str(B.INVALID_ARG) and out[1].split(None, 1)[1] == B.status_string(B.INVALID_ARG)


def test_topk_schedule_is_validated_on_the_host(lib):
    d = (B.ConvDesc * 2)(B.desc(2, 3, 8, 8, 4), B.desc(2, 4, 2, 2, 4))
    m = (ctypes.c_uint8 * 2)(B.APPROX, B.EXACT)
    wsb = lib.conv_wgrad_schedule_topk_workspace_bytes
    assert wsb(d, m, 2, 0) == 0 and wsb(d, m, 2, 65) == 0 and wsb(d, m, 2, 4) > 0
    # a map shorter than topk keeps all of its positions: the 2x2 layer as an approximated one is accepted
    m2 = (ctypes.c_uint8 * 2)(B.APPROX, B.APPROX)
    assert wsb(d, m2, 2, 8) > 0
    vp = ctypes.c_void_p
    one = (vp * 2)(256, 256)
    run = lib.conv_wgrad_schedule_run_topk
    assert run(d, one, one, one, m, 2, 0, 1.0, 1.0, 0, 0, None, 0, None) == B.UNSUPPORTED
    assert run(d, one, one, one, m, 2, 65, 1.0, 1.0, 0, 0, None, 0, None) == B.UNSUPPORTED
    assert run(d, one, one, one, m, 2, 4, 1.0, 1.0, 0, 0, None, 0, None) == B.WORKSPACE_TOO_SMALL
    assert run(d, None, one, one, m, 2, 4, 1.0, 1.0, 0, 0, None, 0, None) == B.INVALID_ARG


def test_topk_schedule_workspace_is_a_slice_per_layer(lib):
    shapes = [(3, 32, 16), (16, 32, 16), (16, 32, 16), (64, 4, 128), (64, 4, 128), (64, 2, 128)]
    descs = [B.desc(8, C, H, H, K) for C, H, K in shapes]
    arr = (B.ConvDesc * len(descs))(*descs)
    m = (ctypes.c_uint8 * len(descs))(*([B.APPROX] * len(descs)))
    for k in (1, 4, 9):
        want = 0
        for d in descs:
            per = B.topk_workspace_bytes(d, min(k, d.Ho * d.Wo))
            want += (per + 255) // 256 * 256
        assert lib.conv_wgrad_schedule_topk_workspace_bytes(arr, m, len(descs), k) == want
