"""CPU-side checks of the C-ABI library: it loads, exports every function
include/bsgd.h declares, and rejects bad arguments on the host before any
GPU work would be enqueued.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_1604_00981_amd as bs
from paper_1604_00981_amd import build as bs_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bsgd.h")
DEBUG_HEADER = os.path.join(ROOT, "include", "bsgd_debug.h")


def _declared_functions(headers=(HEADER, DEBUG_HEADER)):
    names = set()
    for h in headers:
        text = open(h).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(bsgd_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_entry_points():
    names = _declared_functions((HEADER,))
    for must in ("bsgd_step", "bsgd_select_first_n", "bsgd_reduce_update", "bsgd_workspace_bytes",
                 "bsgd_last_status", "bsgd_strerror"):
        assert must in names
    # the product header carries no tuning knob or measurement aid: those live in bsgd_debug.h
    for aid in ("bsgd_set_tuning", "bsgd_set_table_mode", "bsgd_last_launch_count", "bsgd_calibration_copy",
                "bsgd_num_shapes", "bsgd_get_shape"):
        assert aid not in names
        assert aid in _declared_functions((DEBUG_HEADER,))


def test_library_loads_and_exports_every_declared_symbol():
    lib = bs.load_library()
    for name in _declared_functions():
        assert hasattr(lib, name), f"{name} is declared in bsgd.h but not exported"
    assert "gfx950" in bs.bsgd_version()


def test_header_constants_match_binding():
    text = open(HEADER).read()
    consts = dict(re.findall(r"#define\s+(BSGD_[A-Z_]+)\s+\(?(-?\d+)\)?", text))
    for k, v in consts.items():
        assert getattr(bs, k) == int(v), k
    assert ctypes.sizeof(bs.bsgd_hyper) == 32
    assert ctypes.sizeof(bs.bsgd_tensor) == 48


def test_strerror():
    assert bs.strerror(0) == "ok"
    assert "argument" in bs.strerror(bs.BSGD_ERR_ARG)
    assert "fewer than N" in bs.strerror(bs.BSGD_ERR_TOO_FEW)
    assert "unknown" in bs.strerror(-99)


def test_workspace_bytes():
    hy = bs.make_hyper("sgd", 0.1)
    small = bs.bsgd_workspace_bytes(1 << 20, 4, 1, 1, hy)
    assert small >= 256 + 1024 and small % 256 == 0
    hyc = bs.make_hyper("momentum", 0.1, momentum=0.9, clip_norm=1.0)
    big = bs.bsgd_workspace_bytes(1 << 20, 4, 1, 1, hyc)
    assert big >= small + 4 * (1 << 20)            # room for the stored mean gradient
    more_t = bs.bsgd_workspace_bytes(1 << 20, 4, 1, 300, hy)
    assert more_t > small
    for bad in ((-1, 4, 1, 1), (10, 0, 1, 1), (10, 4, -1, 1), (10, 250, 7, 1), (10, 4, 1, 0), (10, 4, 1, 4097)):
        with pytest.raises(bs.BsgdError):
            bs.bsgd_workspace_bytes(*bad, hy)


def test_host_side_argument_checks_enqueue_nothing():
    # raw (fake, never dereferenced on the host) device addresses: every call
    # below must be refused by the host checks
    lib = bs.load_library()
    A = 0x1000                                        # 16-byte and 256-byte aligned
    hy = bs.make_hyper("rmsprop_mom", 0.1, 0.9, 0.9, 1.0)
    tz = bs.make_tensors([(A, A, A, 0, 100)])
    ok_ws = 1 << 20
    # select: N < 1, b < 0, N+b > 256, NULL pointers
    assert lib.bsgd_select_first_n(A, 0, 1, A, A, A, None) == bs.BSGD_ERR_ARG
    assert lib.bsgd_select_first_n(A, 4, -1, A, A, A, None) == bs.BSGD_ERR_ARG
    assert lib.bsgd_select_first_n(A, 250, 7, A, A, A, None) == bs.BSGD_ERR_ARG
    assert lib.bsgd_select_first_n(None, 4, 1, A, A, A, None) == bs.BSGD_ERR_ARG
    assert lib.bsgd_select_first_n(A, 4, 1, None, A, A, None) == bs.BSGD_ERR_ARG
    assert lib.bsgd_select_first_n(A, 4, 1, A, A, None, None) == bs.BSGD_ERR_ARG

    def step(grads=A, ld=100, arr=A, N=4, b=1, tensors=tz, T=1, hyper=hy, ws=A, nbytes=ok_ws):
        return lib.bsgd_step(grads, ld, arr, N, b, tensors, T, ctypes.byref(hyper) if hyper else None, ws, nbytes, None)

    assert step(grads=None) == bs.BSGD_ERR_ARG
    assert step(arr=None) == bs.BSGD_ERR_ARG
    assert step(N=0) == bs.BSGD_ERR_ARG
    assert step(N=256, b=1) == bs.BSGD_ERR_ARG
    assert step(ws=None) == bs.BSGD_ERR_ARG
    assert step(ws=A + 4) == bs.BSGD_ERR_ARG          # workspace not 256-byte aligned
    assert step(nbytes=64) == bs.BSGD_ERR_ARG         # workspace too small
    assert step(hyper=None) == bs.BSGD_ERR_ARG
    assert step(tensors=None) == bs.BSGD_ERR_ARG
    assert step(ld=96) == bs.BSGD_ERR_ARG             # refused before the selection is enqueued
    assert step(ld=102) == bs.BSGD_ERR_ARG

    def ru(grads=A, ld=100, sel=A, N=4, tensors=tz, T=1, hyper=hy, ws=A, nbytes=ok_ws):
        return lib.bsgd_reduce_update(grads, ld, sel, None, N, tensors, T, ctypes.byref(hyper), ws, nbytes, None)

    assert ru(ld=96) == bs.BSGD_ERR_ARG               # row shorter than the tensor
    assert ru(T=0) == bs.BSGD_ERR_ARG
    assert ru(sel=None) == bs.BSGD_ERR_ARG
    assert ru(grads=A + 4) == bs.BSGD_ERR_ARG         # gradient base not 16-byte aligned
    assert ru(ld=102) == bs.BSGD_ERR_ARG              # row stride not a multiple of 4 elements
    assert ru(nbytes=1024) == bs.BSGD_ERR_ARG
    assert ru(hyper=bs.make_hyper(7, 0.1)) == bs.BSGD_ERR_ARG          # unknown optimizer
    no_s1 = bs.make_tensors([(A, A, None, 0, 100)])
    assert ru(tensors=no_s1) == bs.BSGD_ERR_ARG       # RMSProp needs both state buffers
    no_s0 = bs.make_tensors([(A, None, None, 0, 100)])
    assert ru(tensors=no_s0, hyper=bs.make_hyper("momentum", 0.1, 0.9)) == bs.BSGD_ERR_ARG
    neg = bs.make_tensors([(A, A, A, -4, 100)])
    assert ru(tensors=neg) == bs.BSGD_ERR_ARG
    odd = bs.make_tensors([(A + 2, A, A, 0, 100)])
    assert ru(tensors=odd) == bs.BSGD_ERR_ARG         # theta not 4-byte aligned
    # two tensors may not claim the same gradient columns (whatever order they are listed in)
    big_ws = 1 << 22
    clash = bs.make_tensors([(A, A, A, 50, 100), (A, A, A, 0, 51)])
    assert ru(tensors=clash, T=2, ld=152, nbytes=big_ws) == bs.BSGD_ERR_ARG
    # a moving average on some tensors only, or a decay outside [0,1], is refused
    some = bs.make_tensors([(A, A, A, 0, 50, A), (A, A, A, 50, 50)])
    assert ru(tensors=some, T=2, nbytes=big_ws) == bs.BSGD_ERR_ARG
    alle = bs.make_tensors([(A, A, A, 0, 100, A)])
    assert ru(tensors=alle, hyper=bs.make_hyper("rmsprop_mom", 0.1, 0.9, 0.9, 1.0, ema_decay=1.5)) == bs.BSGD_ERR_ARG
    # selection options: NaN deadline, n_min out of range
    so = bs.make_select_opts(None, 0, float('nan'), 0)
    assert lib.bsgd_select_ex(A, 4, 1, ctypes.byref(so), A, A, A, A, None) == bs.BSGD_ERR_ARG
    so = bs.make_select_opts(None, 0, 1.0, 6)
    assert lib.bsgd_select_ex(A, 4, 1, ctypes.byref(so), A, A, A, A, None) == bs.BSGD_ERR_ARG
    so = bs.make_select_opts(None, 0, 1.0, 2)
    assert lib.bsgd_select_ex(A, 4, 1, ctypes.byref(so), A, None, A, A, None) == bs.BSGD_ERR_ARG   # count needed
    assert lib.bsgd_step_ex(A, 100, A, 4, 1, None, tz, 1, ctypes.byref(hy), A, ok_ws, None) == bs.BSGD_ERR_ARG
    # clipping needs the larger workspace
    hyc = bs.make_hyper("sgd", 0.1, clip_norm=1.0)
    need = bs.bsgd_workspace_bytes(100, 4, 1, 1, hyc)
    assert ru(hyper=hyc, nbytes=need - 256) == bs.BSGD_ERR_ARG


def test_tuning_rejects_unknown_shapes():
    with pytest.raises(bs.BsgdError):
        bs.bsgd_set_tuning(192, 3, 7, 1)
    bs.bsgd_set_tuning()                              # keep current
    n = bs.bsgd_num_shapes()
    assert n >= 1
    shapes = [bs.bsgd_get_shape(i) for i in range(n)]
    assert len(set(shapes)) == n
    for blk, vec, unroll, nt in shapes:
        assert blk % 64 == 0 and vec >= 1 and unroll >= 1 and nt in (0, 1)
    with pytest.raises(bs.BsgdError):
        bs.bsgd_get_shape(n)


def test_table_mode_accepts_only_known_modes():
    with pytest.raises(bs.BsgdError):
        bs.bsgd_set_table_mode(2)
    with pytest.raises(bs.BsgdError):
        bs.bsgd_set_table_mode(-1)
    bs.bsgd_set_table_mode(1)
    bs.bsgd_set_table_mode(0)


def test_build_sources_exist():
    for p in bs_build.SOURCES + bs_build.HEADERS:
        assert os.path.exists(p)


def test_header_is_plain_c_and_struct_layouts_match_the_binding(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with a C
    compiler, and a C program must see the struct layouts the binding uses."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stddef.h>\n#include <stdio.h>\n#include "bsgd.h"\n#include "bsgd_debug.h"\n'
        "int main(void) {\n"
        '  printf("hyper %zu", sizeof(bsgd_hyper));\n'
        + "".join(f'  printf(" %zu", offsetof(bsgd_hyper, {f}));\n' for f, _ in bs.bsgd_hyper._fields_)
        + '  printf("\\ntensor %zu", sizeof(bsgd_tensor));\n'
        + "".join(f'  printf(" %zu", offsetof(bsgd_tensor, {f}));\n' for f, _ in bs.bsgd_tensor._fields_)
        + '  printf("\\nopts %zu", sizeof(bsgd_select_opts));\n'
        + "".join(f'  printf(" %zu", offsetof(bsgd_select_opts, {f}));\n' for f, _ in bs.bsgd_select_opts._fields_)
        + '  printf("\\n");\n  return 0;\n}\n')
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout.split("\n")
    for line, st in zip(out, (bs.bsgd_hyper, bs.bsgd_tensor, bs.bsgd_select_opts)):
        nums = [int(x) for x in line.split()[1:]]
        assert nums[0] == ctypes.sizeof(st), line
        assert nums[1:] == [getattr(st, f).offset for f, _ in st._fields_], line
