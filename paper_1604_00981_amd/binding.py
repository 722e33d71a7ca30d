"""ctypes binding of libbsgd.so: same names as the C entry points in
include/bsgd.h, argument marshalling only.  Every step of the path runs in
the HIP kernels; there is no CPU fallback, and a missing library is an error.

PyTorch is used for device memory and streams: arguments are CUDA/HIP
tensors (or raw device addresses as ints) and the launch goes to torch's
current stream unless one is given.
"""
from __future__ import annotations

import ctypes
import os
from typing import Iterable, List, Optional, Sequence, Tuple, Union

import torch  # imported before the library so both share one HIP runtime

from . import build as _build

BSGD_OK = 0
BSGD_ERR_ARG = -1
BSGD_ERR_TOO_FEW = -2
BSGD_ERR_HIP = -3
BSGD_ERR_SCRATCH = -4
BSGD_STATIC_SCRATCH_BYTES = 33554432
BSGD_MAX_WORKERS = 256
BSGD_MAX_TENSORS = 4096

BSGD_SGD, BSGD_MOMENTUM, BSGD_RMSPROP_MOM = 0, 1, 2
_OPT_BY_NAME = {"sgd": BSGD_SGD, "momentum": BSGD_MOMENTUM, "rmsprop_mom": BSGD_RMSPROP_MOM}


class bsgd_hyper(ctypes.Structure):
    _fields_ = [("opt", ctypes.c_int32), ("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("decay", ctypes.c_float), ("eps", ctypes.c_float), ("clip_norm", ctypes.c_float),
                ("ema_decay", ctypes.c_float), ("worker_clip_norm", ctypes.c_float)]


class bsgd_tensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("s0", ctypes.c_void_p), ("s1", ctypes.c_void_p),
                ("grad_offset", ctypes.c_int64), ("numel", ctypes.c_int64), ("ema", ctypes.c_void_p)]


class bsgd_select_opts(ctypes.Structure):
    _fields_ = [("tags", ctypes.c_void_p), ("step_tag", ctypes.c_int32), ("deadline", ctypes.c_float),
                ("n_min", ctypes.c_int32), ("row_count", ctypes.c_void_p)]


class BsgdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libbsgd.so (building it first only when no built library exists)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _build.LIB_PATH
    if not os.path.exists(p):
        if path is not None:
            raise FileNotFoundError(p)
        _build.build_library(verbose=False)
    lib = ctypes.CDLL(p)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.bsgd_select_first_n.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.bsgd_select_first_n.restype = ctypes.c_int
    lib.bsgd_reduce_update.argtypes = [vp, i64, vp, vp, i32, ctypes.POINTER(bsgd_tensor), i32,
                                       ctypes.POINTER(bsgd_hyper), vp, sz, vp]
    lib.bsgd_reduce_update.restype = ctypes.c_int
    lib.bsgd_step.argtypes = [vp, i64, vp, i32, i32, ctypes.POINTER(bsgd_tensor), i32,
                              ctypes.POINTER(bsgd_hyper), vp, sz, vp]
    lib.bsgd_step.restype = ctypes.c_int
    lib.bsgd_step_noalloc.argtypes = [vp, i64, vp, i32, i32, ctypes.POINTER(bsgd_tensor), i32,
                                      ctypes.POINTER(bsgd_hyper), vp, vp, vp]
    lib.bsgd_step_noalloc.restype = ctypes.c_int
    lib.bsgd_select_ex.argtypes = [vp, i32, i32, ctypes.POINTER(bsgd_select_opts), vp, vp, vp, vp, vp]
    lib.bsgd_select_ex.restype = ctypes.c_int
    lib.bsgd_step_ex.argtypes = [vp, i64, vp, i32, i32, ctypes.POINTER(bsgd_select_opts), ctypes.POINTER(bsgd_tensor), i32,
                                 ctypes.POINTER(bsgd_hyper), vp, sz, vp]
    lib.bsgd_step_ex.restype = ctypes.c_int
    lib.bsgd_last_kept_count.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.bsgd_last_kept_count.restype = ctypes.c_int
    lib.bsgd_workspace_bytes.argtypes = [i64, i32, i32, i32, ctypes.POINTER(bsgd_hyper)]
    lib.bsgd_workspace_bytes.restype = sz
    lib.bsgd_last_status.argtypes = [vp, vp, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_float)]
    lib.bsgd_last_status.restype = ctypes.c_int
    lib.bsgd_last_selection.argtypes = [vp, vp, i32, ctypes.POINTER(i32)]
    lib.bsgd_last_selection.restype = ctypes.c_int
    lib.bsgd_last_clip.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)]
    lib.bsgd_last_clip.restype = ctypes.c_int
    lib.bsgd_set_tuning.argtypes = [i32, i32, i32, i32]
    lib.bsgd_set_tuning.restype = ctypes.c_int
    lib.bsgd_set_table_mode.argtypes = [i32]
    lib.bsgd_set_table_mode.restype = ctypes.c_int
    lib.bsgd_last_launch_count.argtypes = []
    lib.bsgd_last_launch_count.restype = ctypes.c_int
    lib.bsgd_debug_chunk_runs.argtypes = [ctypes.POINTER(bsgd_tensor), i32, i64, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                          i32, ctypes.POINTER(i32)]
    lib.bsgd_debug_chunk_runs.restype = ctypes.c_int
    lib.bsgd_set_fused_selection.argtypes = [i32]
    lib.bsgd_set_fused_selection.restype = ctypes.c_int
    lib.bsgd_last_step_fused_selection.argtypes = []
    lib.bsgd_last_step_fused_selection.restype = ctypes.c_int
    lib.bsgd_num_shapes.argtypes = []
    lib.bsgd_num_shapes.restype = ctypes.c_int
    lib.bsgd_get_shape.argtypes = [i32, ctypes.POINTER(i32)]
    lib.bsgd_get_shape.restype = ctypes.c_int
    lib.bsgd_calibration_copy.argtypes = [vp, vp, i64, vp]
    lib.bsgd_calibration_copy.restype = ctypes.c_int
    lib.bsgd_yardstick_streams.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(vp), i32, i64, i32, vp]
    lib.bsgd_yardstick_streams.restype = ctypes.c_int
    lib.bsgd_last_gradient_count.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.bsgd_last_gradient_count.restype = ctypes.c_int
    lib.bsgd_precombine.argtypes = [vp, i64, i64, vp, ctypes.POINTER(i32), i32, vp, i64, vp, vp, vp]
    lib.bsgd_precombine.restype = ctypes.c_int
    lib.bsgd_straggler_workspace_bytes.argtypes = [i32, i64]
    lib.bsgd_straggler_workspace_bytes.restype = sz
    lib.bsgd_kth_arrival_times.argtypes = [vp, i32, i64, vp, vp, vp, sz, vp]
    lib.bsgd_kth_arrival_times.restype = ctypes.c_int
    dp = ctypes.POINTER(ctypes.c_double)
    lib.bsgd_time_to_converge.argtypes = [dp, i32, dp, dp, i32, dp, ctypes.POINTER(i32)]
    lib.bsgd_time_to_converge.restype = ctypes.c_int
    lib.bsgd_strerror.argtypes = [ctypes.c_int]
    lib.bsgd_strerror.restype = ctypes.c_char_p
    lib.bsgd_version.argtypes = []
    lib.bsgd_version.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


# ----------------------------------------------------------------------------
# marshalling helpers
# ----------------------------------------------------------------------------
DevPtr = Union[torch.Tensor, int, None]


def _ptr(x: DevPtr, dtype: Optional[torch.dtype] = None, name: str = "arg") -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not isinstance(x, torch.Tensor):
        raise TypeError(f"{name}: expected a device tensor or an address")
    if not x.is_cuda:
        raise ValueError(f"{name}: must live on the GPU")
    if dtype is not None and x.dtype != dtype:
        raise ValueError(f"{name}: expected {dtype}, got {x.dtype}")
    if not x.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_hyper(opt, lr: float, momentum: float = 0.0, decay: float = 0.0, eps: float = 0.0,
               clip_norm: float = 0.0, ema_decay: float = 0.0, worker_clip_norm: float = 0.0) -> bsgd_hyper:
    code = _OPT_BY_NAME[opt] if isinstance(opt, str) else int(opt)
    return bsgd_hyper(code, lr, momentum, decay, eps, clip_norm, ema_decay, worker_clip_norm)


def make_tensors(items: Iterable[Tuple[DevPtr, DevPtr, DevPtr, int, int]]):
    """ctypes array of bsgd_tensor from (theta, s0, s1, grad_offset, numel[, ema])."""
    items = list(items)
    arr = (bsgd_tensor * len(items))()
    for d, item in zip(arr, items):
        theta, s0, s1, off, numel = item[:5]
        d.theta = _ptr(theta, torch.float32, "theta")
        d.s0 = _ptr(s0, torch.float32, "s0")
        d.s1 = _ptr(s1, torch.float32, "s1")
        d.grad_offset = int(off)
        d.numel = int(numel)
        d.ema = _ptr(item[5], torch.float32, "ema") if len(item) > 5 else None
    return arr


def make_select_opts(tags: DevPtr = None, step_tag: int = 0, deadline: float = float("inf"), n_min: int = 0,
                     row_count: DevPtr = None):
    """bsgd_select_opts; keep the tags / row_count tensors alive as long as the struct is used."""
    return bsgd_select_opts(_ptr(tags, torch.int32, "tags"), step_tag, deadline, n_min,
                            _ptr(row_count, torch.int32, "row_count"))


def _check(rc: int, where: str) -> None:
    if rc != BSGD_OK:
        raise BsgdError(rc, where)


# ----------------------------------------------------------------------------
# entry points (same names as the C ABI)
# ----------------------------------------------------------------------------
def bsgd_select_first_n(arrival_t: DevPtr, N: int, b: int, sel_idx: DevPtr, t_step: DevPtr, status: DevPtr,
                        stream=None) -> None:
    lib = load_library()
    _check(lib.bsgd_select_first_n(_ptr(arrival_t, torch.float32, "arrival_t"), N, b,
                                   _ptr(sel_idx, torch.int32, "sel_idx"), _ptr(t_step, torch.float32, "t_step"),
                                   _ptr(status, torch.int32, "status"), _stream(stream)), "bsgd_select_first_n")


def bsgd_select_ex(arrival_t: DevPtr, N: int, b: int, opts: bsgd_select_opts, sel_idx: DevPtr, n_kept: DevPtr,
                   t_step: DevPtr, status: DevPtr, stream=None) -> None:
    lib = load_library()
    _check(lib.bsgd_select_ex(_ptr(arrival_t, torch.float32, "arrival_t"), N, b, ctypes.byref(opts),
                              _ptr(sel_idx, torch.int32, "sel_idx"), _ptr(n_kept, torch.int32, "n_kept"),
                              _ptr(t_step, torch.float32, "t_step"), _ptr(status, torch.int32, "status"),
                              _stream(stream)), "bsgd_select_ex")


def _ws(workspace: DevPtr, workspace_bytes: Optional[int]) -> Tuple[int, int]:
    if isinstance(workspace, torch.Tensor):
        n = workspace.numel() * workspace.element_size()
        return _ptr(workspace, None, "workspace"), n if workspace_bytes is None else workspace_bytes
    if workspace_bytes is None:
        raise ValueError("workspace_bytes is required with a raw workspace address")
    return workspace, workspace_bytes


def bsgd_reduce_update(grads: DevPtr, ld: int, sel_idx: DevPtr, status: DevPtr, N: int, tensors, hyper: bsgd_hyper,
                       workspace: DevPtr, workspace_bytes: Optional[int] = None, stream=None) -> None:
    lib = load_library()
    ws, nbytes = _ws(workspace, workspace_bytes)
    _check(lib.bsgd_reduce_update(_ptr(grads, torch.float32, "grads"), ld, _ptr(sel_idx, torch.int32, "sel_idx"),
                                  _ptr(status, torch.int32, "status"), N, tensors, len(tensors),
                                  ctypes.byref(hyper), ws, nbytes, _stream(stream)), "bsgd_reduce_update")


def bsgd_step(grads: DevPtr, ld: int, arrival_t: DevPtr, N: int, b: int, tensors, hyper: bsgd_hyper,
              workspace: DevPtr, workspace_bytes: Optional[int] = None, stream=None) -> None:
    lib = load_library()
    ws, nbytes = _ws(workspace, workspace_bytes)
    _check(lib.bsgd_step(_ptr(grads, torch.float32, "grads"), ld, _ptr(arrival_t, torch.float32, "arrival_t"),
                         N, b, tensors, len(tensors), ctypes.byref(hyper), ws, nbytes, _stream(stream)), "bsgd_step")


def bsgd_step_noalloc(grads: DevPtr, ld: int, arrival_t: DevPtr, N: int, b: int, tensors, hyper: bsgd_hyper,
                      status: DevPtr, t_step: DevPtr = None, stream=None) -> None:
    """bsgd_step on the library's own static device scratch (no workspace argument, nothing allocated)."""
    lib = load_library()
    _check(lib.bsgd_step_noalloc(_ptr(grads, torch.float32, "grads"), ld, _ptr(arrival_t, torch.float32, "arrival_t"),
                                 N, b, tensors, len(tensors), ctypes.byref(hyper), _ptr(status, torch.int32, "status"),
                                 _ptr(t_step, torch.float32, "t_step"), _stream(stream)), "bsgd_step_noalloc")


def bsgd_step_ex(grads: DevPtr, ld: int, arrival_t: DevPtr, N: int, b: int, opts: bsgd_select_opts, tensors,
                 hyper: bsgd_hyper, workspace: DevPtr, workspace_bytes: Optional[int] = None, stream=None) -> None:
    lib = load_library()
    ws, nbytes = _ws(workspace, workspace_bytes)
    _check(lib.bsgd_step_ex(_ptr(grads, torch.float32, "grads"), ld, _ptr(arrival_t, torch.float32, "arrival_t"),
                            N, b, ctypes.byref(opts), tensors, len(tensors), ctypes.byref(hyper), ws, nbytes,
                            _stream(stream)), "bsgd_step_ex")


def bsgd_last_kept_count(workspace: DevPtr, stream=None) -> int:
    n = ctypes.c_int32(0)
    _check(load_library().bsgd_last_kept_count(_ptr(workspace, None, "workspace"), _stream(stream), ctypes.byref(n)),
           "bsgd_last_kept_count")
    return n.value


def bsgd_workspace_bytes(span: int, N: int, b: int, T: int, hyper: bsgd_hyper) -> int:
    n = load_library().bsgd_workspace_bytes(span, N, b, T, ctypes.byref(hyper))
    if n == 0:
        raise BsgdError(BSGD_ERR_ARG, "bsgd_workspace_bytes")
    return n


def bsgd_last_status(workspace: DevPtr, stream=None) -> Tuple[int, float]:
    st, ts = ctypes.c_int32(0), ctypes.c_float(0.0)
    _check(load_library().bsgd_last_status(_ptr(workspace, None, "workspace"), _stream(stream),
                                           ctypes.byref(st), ctypes.byref(ts)), "bsgd_last_status")
    return st.value, ts.value


def bsgd_last_selection(workspace: DevPtr, N: int, stream=None) -> List[int]:
    out = (ctypes.c_int32 * N)()
    _check(load_library().bsgd_last_selection(_ptr(workspace, None, "workspace"), _stream(stream), N, out),
           "bsgd_last_selection")
    return list(out)


def bsgd_last_clip(workspace: DevPtr, stream=None) -> Tuple[float, float]:
    nrm, sc = ctypes.c_double(0.0), ctypes.c_float(0.0)
    _check(load_library().bsgd_last_clip(_ptr(workspace, None, "workspace"), _stream(stream),
                                         ctypes.byref(nrm), ctypes.byref(sc)), "bsgd_last_clip")
    return nrm.value, sc.value


def bsgd_set_table_mode(mode: int = 0) -> None:
    """0: launches carry their part of the tensor table as an argument when it fits; 1: always via the workspace."""
    _check(load_library().bsgd_set_table_mode(mode), "bsgd_set_table_mode")


def bsgd_set_tuning(block: int = -1, vec: int = -1, unroll: int = -1, nontemporal: int = -1) -> None:
    _check(load_library().bsgd_set_tuning(block, vec, unroll, nontemporal), "bsgd_set_tuning")


def bsgd_last_launch_count() -> int:
    return load_library().bsgd_last_launch_count()


def bsgd_debug_chunk_runs(tensors, chunk_cols: int, capacity: int = 8192) -> List[Tuple[int, int]]:
    """(first chunk, chunk count) of every run of chunks a call with these tensors launches (host logic only)."""
    first = (ctypes.c_int64 * capacity)()
    count = (ctypes.c_int64 * capacity)()
    n = ctypes.c_int32(0)
    _check(load_library().bsgd_debug_chunk_runs(tensors, len(tensors), chunk_cols, first, count, capacity, ctypes.byref(n)),
           "bsgd_debug_chunk_runs")
    return [(int(first[i]), int(count[i])) for i in range(n.value)]


def bsgd_set_fused_selection(on: bool = True) -> None:
    _check(load_library().bsgd_set_fused_selection(1 if on else 0), "bsgd_set_fused_selection")


def bsgd_last_step_fused_selection() -> bool:
    return bool(load_library().bsgd_last_step_fused_selection())


def bsgd_num_shapes() -> int:
    return load_library().bsgd_num_shapes()


def bsgd_get_shape(i: int) -> Tuple[int, int, int, int]:
    out = (ctypes.c_int32 * 4)()
    _check(load_library().bsgd_get_shape(i, out), "bsgd_get_shape")
    return tuple(out)


def bsgd_calibration_copy(dst: DevPtr, src: DevPtr, nbytes: int, stream=None) -> None:
    _check(load_library().bsgd_calibration_copy(_ptr(dst, None, "dst"), _ptr(src, None, "src"), nbytes,
                                                _stream(stream)), "bsgd_calibration_copy")


def bsgd_yardstick_streams(reads: Sequence[DevPtr], writes: Sequence[DevPtr], nbytes: int, vec: int = 8, stream=None) -> None:
    """Plain streaming kernel over len(reads) read and len(writes) written buffers of nbytes each (measurement aid)."""
    rd = (ctypes.c_void_p * max(len(reads), 1))(*[_ptr(x, None, "read") for x in reads])
    wr = (ctypes.c_void_p * max(len(writes), 1))(*[_ptr(x, None, "write") for x in writes])
    _check(load_library().bsgd_yardstick_streams(rd, len(reads), wr, len(writes), nbytes, vec, _stream(stream)),
           "bsgd_yardstick_streams")


def bsgd_last_gradient_count(workspace: torch.Tensor, stream=None) -> int:
    out = ctypes.c_int32(0)
    _check(load_library().bsgd_last_gradient_count(_ptr(workspace, None, "workspace"), _stream(stream),
                                                   ctypes.byref(out)), "bsgd_last_gradient_count")
    return int(out.value)


def bsgd_precombine(grads: DevPtr, ld: int, cols: int, arrival_t: DevPtr, group_size: Sequence[int],
                    combined: DevPtr, ld_out: int, arrival_m: DevPtr, row_count: DevPtr, stream=None) -> None:
    """Sec. 6: one message per machine = the sum of its workers' gradient rows."""
    M = len(group_size)
    gs = (ctypes.c_int32 * max(M, 1))(*[int(g) for g in group_size])
    _check(load_library().bsgd_precombine(
        _ptr(grads, torch.float32, "grads"), ld, cols, _ptr(arrival_t, torch.float32, "arrival_t"), gs, M,
        _ptr(combined, torch.float32, "combined"), ld_out, _ptr(arrival_m, torch.float32, "arrival_m"),
        _ptr(row_count, torch.int32, "row_count"), _stream(stream)), "bsgd_precombine")


def bsgd_straggler_workspace_bytes(W: int, B: int) -> int:
    return int(load_library().bsgd_straggler_workspace_bytes(W, B))


def bsgd_kth_arrival_times(arrival_t: DevPtr, W: int, B: int, kth_time: Optional[DevPtr], mean_kth: Optional[DevPtr],
                           workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Sec. 3.1: per iteration, the time to collect k gradients (rows of
    arrival_t in ascending order) and/or their mean over iterations."""
    _check(load_library().bsgd_kth_arrival_times(
        _ptr(arrival_t, torch.float32, "arrival_t"), W, B,
        _ptr(kth_time, torch.float32, "kth_time") if kth_time is not None else None,
        _ptr(mean_kth, torch.float64, "mean_kth") if mean_kth is not None else None,
        _ptr(workspace, None, "workspace") if workspace is not None else None,
        workspace.numel() * workspace.element_size() if workspace is not None else 0,
        _stream(stream)), "bsgd_kth_arrival_times")


def bsgd_time_to_converge(mean_kth: Sequence[float], measured: Sequence[Tuple[float, float]]):
    """Sec. 3.1: (est[W], best_N) from the mean time to collect k gradients
    and measured (N, iterations) points; host arithmetic inside the library."""
    W = len(mean_kth)
    m = (ctypes.c_double * W)(*[float(x) for x in mean_kth])
    n = len(measured)
    mn = (ctypes.c_double * max(n, 1))(*[float(p[0]) for p in measured])
    mi = (ctypes.c_double * max(n, 1))(*[float(p[1]) for p in measured])
    est = (ctypes.c_double * W)()
    best = ctypes.c_int32(0)
    _check(load_library().bsgd_time_to_converge(m, W, mn, mi, n, est, ctypes.byref(best)), "bsgd_time_to_converge")
    return list(est), int(best.value)


def strerror(code: int) -> str:
    return load_library().bsgd_strerror(code).decode()


def bsgd_version() -> str:
    return load_library().bsgd_version().decode()


def alloc_workspace(span: int, N: int, b: int, T: int, hyper: bsgd_hyper, device="cuda") -> torch.Tensor:
    """A torch uint8 buffer of the size the library asks for (torch's caching
    allocator hands out 512-byte aligned blocks)."""
    n = bsgd_workspace_bytes(span, N, b, T, hyper)
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    assert ws.data_ptr() % 256 == 0
    return ws
