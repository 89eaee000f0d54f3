"""ctypes binding of libddp_gfx950.so.

One Python function per C entry point of include/ddp_gfx950.h, with the same
name.  The functions only marshal arguments (lists / numpy arrays -> C arrays)
and turn negative status codes into DdpError; every step of the path runs in
the library's HIP kernels.  There is no fallback: if the shared library has not
been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

# The process must hold a single HIP runtime.  PyTorch ships its own copy of
# libamdhip64 under the same SONAME; importing torch first makes the dynamic
# linker resolve this library's dependency to that already-loaded copy, so that
# the stream handles torch hands out are valid inside the library.
try:  # pragma: no cover - torch is present wherever a GPU is used
    import torch  # noqa: F401
except Exception:  # torch missing: the system runtime is used
    pass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libddp_gfx950.so")

DDP_OK = 0
DDP_ERR_ARG, DDP_ERR_STATE, DDP_ERR_ALREADY_READY = -1, -2, -3
DDP_ERR_HIP, DDP_ERR_NO_DEVICE, DDP_ERR_UNSUPPORTED = -4, -5, -6
DDP_FP32, DDP_FP16, DDP_BF16 = 0, 1, 2
DDP_MAX_REPLICAS = 64
DDP_DEVICE_NONE = -1
DDP_CAP_WHOLE_MODEL = (1 << 64) - 1
DDP_OPT_PIPELINE, DDP_OPT_WRITE_ALL, DDP_OPT_TIMING = 1, 2, 3
DDP_OPT_NONTEMPORAL = 5
DDP_OPT_EMIT_BUSY_BLOCKS = 8
DDP_OPT_COALESCE, DDP_OPT_FIND_UNUSED, DDP_OPT_REDUCE_STREAMS = 10, 11, 12
DDP_OPT_REDUCE_BLOCKS_PER_CU, DDP_OPT_REDUCE_CAP_MIN_BYTES = 13, 14
DDP_OPT_ACCUMULATE_BLOCKS_PER_CU, DDP_OPT_TAIL_ON_BACKWARD = 16, 17
DDP_OPT_FLAG_ORDER, DDP_OPT_GATE_WAIT_US, DDP_OPT_LAUNCH_HOLD, DDP_OPT_CHAIN_LAUNCHES = 18, 19, 21, 22
DDP_STAT_REPAIRED_LAUNCHES = 100
DDP_PIPELINE_STAGED, DDP_PIPELINE_FUSED = 0, 1
DDP_STATIC_SCRATCH_BYTES = 32 << 20
DDP_K_PACK, DDP_K_REDUCE, DDP_K_UNPACK, DDP_K_ACCUMULATE, DDP_K_ITERATION = 0, 1, 2, 3, 4

EXPORTS = [
    "ddp_version", "ddp_last_error", "ddp_create", "ddp_destroy", "ddp_set_option", "ddp_get_option",
    "ddp_register_params", "ddp_set_outputs", "ddp_build_buckets", "ddp_rebuild_buckets", "ddp_get_ready_order",
    "ddp_get_assignment",
    "ddp_get_bucket_info", "ddp_get_bucket_ptr", "ddp_mark_ready", "ddp_mark_ready_local",
    "ddp_get_global_used",
    "ddp_mark_ready_many", "ddp_finalize_backward", "ddp_synchronize",
    "ddp_get_launch_log", "ddp_no_sync_accumulate", "ddp_get_used_map",
    "ddp_synth_backward", "ddp_get_kernel_times", "ddp_sync_static",
]


class DdpError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"ddp error {code}: {message}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python paper_2006_15704_amd/build.py` "
        "(there is no fallback implementation)")

_lib = C.CDLL(LIB_PATH)


def _refuse_stale_library() -> None:
    """The library carries a digest of the sources it was compiled from; if the
    sources next to it have changed since, results would silently describe old
    code."""
    from . import build as _build
    _lib.ddp_version.restype = C.c_char_p
    have = _lib.ddp_version().decode().rsplit("ddp-src-hash:", 1)[-1]
    want = _build.source_hash()
    if have != want:
        raise ImportError(
            f"{LIB_PATH} was built from other sources (digest {have}, sources on disk {want}): "
            "rebuild it with `python paper_2006_15704_amd/build.py`")


_refuse_stale_library()

_vp, _i32, _i64, _u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
_lib.ddp_version.restype = C.c_char_p
_lib.ddp_last_error.restype = C.c_char_p
_lib.ddp_last_error.argtypes = [_vp]
_lib.ddp_create.argtypes = [C.POINTER(_vp), _i32, _i32, _vp, _vp]
_lib.ddp_destroy.argtypes = [_vp]
_lib.ddp_set_option.argtypes = [_vp, _i32, _i64]
_lib.ddp_get_option.argtypes = [_vp, _i32, C.POINTER(_i64)]
_lib.ddp_register_params.argtypes = [_vp, _i32, C.POINTER(_i64), C.POINTER(_i32), C.POINTER(_vp)]
_lib.ddp_set_outputs.argtypes = [_vp, C.POINTER(_vp)]
_lib.ddp_build_buckets.argtypes = [_vp, _u64]
_lib.ddp_rebuild_buckets.argtypes = [_vp, _u64]
_lib.ddp_get_ready_order.argtypes = [_vp, _i32, C.POINTER(_i32), _i32, C.POINTER(_i32)]
_lib.ddp_get_assignment.argtypes = [_vp, C.POINTER(_i32), C.POINTER(_i64)]
_lib.ddp_get_bucket_info.argtypes = [_vp, _i32, C.POINTER(_i64), C.POINTER(_i32), C.POINTER(_i32)]
_lib.ddp_get_bucket_ptr.argtypes = [_vp, _i32, _i32, C.POINTER(_vp)]
_lib.ddp_mark_ready.argtypes = [_vp, _i32]
_lib.ddp_mark_ready_local.argtypes = [_vp, _i32, C.POINTER(C.c_uint8)]
_lib.ddp_get_global_used.argtypes = [_vp, C.POINTER(C.c_uint8)]
_lib.ddp_mark_ready_many.argtypes = [_vp, C.POINTER(_i32), _i32]
_lib.ddp_finalize_backward.argtypes = [_vp]
_lib.ddp_synchronize.argtypes = [_vp]
_lib.ddp_get_launch_log.argtypes = [_vp, _i32, C.POINTER(_i32), C.POINTER(_i32), _i32, C.POINTER(_i32)]
_lib.ddp_no_sync_accumulate.argtypes = [_vp, C.POINTER(_vp)]
_lib.ddp_get_used_map.argtypes = [_vp, _i32, C.POINTER(C.c_uint8)]
_lib.ddp_synth_backward.argtypes = [_vp, C.POINTER(_i32), _i32, C.POINTER(_i64), C.POINTER(_vp), _i32]
_lib.ddp_get_kernel_times.argtypes = [_vp, _i32, C.POINTER(C.c_float), C.POINTER(_i32), _i32, C.POINTER(_i32)]
_lib.ddp_sync_static.argtypes = [_i32, _i32, _vp, _i32, C.POINTER(_i64), C.POINTER(_i32), C.POINTER(_vp), _u64]
for _name in EXPORTS:
    if _name not in ("ddp_version", "ddp_last_error"):
        getattr(_lib, _name).restype = _i32


def _check(ctx, status: int) -> int:
    if status < 0:
        msg = _lib.ddp_last_error(ctx)
        raise DdpError(status, msg.decode() if msg else "")
    return status


def _i32_array(values) -> np.ndarray:
    return np.ascontiguousarray(values, dtype=np.int32)


def _i64_array(values) -> np.ndarray:
    return np.ascontiguousarray(values, dtype=np.int64)


def _ptr_array(values) -> np.ndarray:
    """Device addresses (ints, None = NULL) -> contiguous uint64 array."""
    return np.ascontiguousarray([0 if v is None else int(v) for v in values], dtype=np.uint64)


def _as(arr: np.ndarray, ctype):
    return arr.ctypes.data_as(C.POINTER(ctype))


def ddp_version() -> str:
    return _lib.ddp_version().decode()


def ddp_last_error(ctx) -> str:
    msg = _lib.ddp_last_error(ctx)
    return msg.decode() if msg else ""


_replicas = {}      # context address -> R, for checking array lengths before they cross the C ABI
_nparams = {}       # context address -> n


def ddp_create(R: int, device: int, reduce_stream: int = 0, backward_stream: int = 0):
    """Returns the opaque context handle.  Streams are raw hipStream_t values
    (torch.cuda.Stream.cuda_stream)."""
    handle = _vp()
    _check(None, _lib.ddp_create(C.byref(handle), R, device, _vp(reduce_stream or None),
                                 _vp(backward_stream or None)))
    _replicas[handle.value] = int(R)
    return handle


def ddp_destroy(ctx) -> None:
    _replicas.pop(ctx.value, None)
    _nparams.pop(ctx.value, None)
    _check(ctx, _lib.ddp_destroy(ctx))


def ddp_set_option(ctx, option: int, value: int) -> None:
    _check(ctx, _lib.ddp_set_option(ctx, option, value))


def ddp_get_option(ctx, option: int) -> int:
    value = _i64()
    _check(ctx, _lib.ddp_get_option(ctx, option, C.byref(value)))
    return value.value


def ddp_register_params(ctx, numel: Sequence[int], dtype: Sequence[int],
                        grad_ptrs: Optional[Sequence[int]]) -> None:
    """grad_ptrs: flat sequence of R*n device addresses, [r][i] row-major."""
    ne, dt = _i64_array(numel), _i32_array(dtype)
    if grad_ptrs is None:
        gp = None
    else:
        arr = _ptr_array(grad_ptrs)
        gp = _as(arr, _vp)
    _check(ctx, _lib.ddp_register_params(ctx, len(ne), _as(ne, _i64), _as(dt, _i32), gp))
    _nparams[ctx.value] = len(ne)


def ddp_set_outputs(ctx, out_ptrs: Optional[Sequence[int]]) -> None:
    """out_ptrs: n device addresses of binary32 tensors that receive the averages."""
    if out_ptrs is None:
        _check(ctx, _lib.ddp_set_outputs(ctx, None))
        return
    arr = _ptr_array(out_ptrs)
    if len(arr) != _nparams.get(ctx.value, len(arr)):      # the library reads exactly n pointers
        raise ValueError(f"out_ptrs has {len(arr)} entries, {_nparams[ctx.value]} parameters are registered")
    _check(ctx, _lib.ddp_set_outputs(ctx, _as(arr, _vp)))


def ddp_build_buckets(ctx, cap_bytes: int) -> int:
    return _check(ctx, _lib.ddp_build_buckets(ctx, cap_bytes))


def ddp_get_assignment(ctx, n: int):
    bucket_of = np.zeros(n, dtype=np.int32)
    offset = np.zeros(n, dtype=np.int64)
    _check(ctx, _lib.ddp_get_assignment(ctx, _as(bucket_of, _i32), _as(offset, _i64)))
    return bucket_of, offset


def ddp_get_bucket_info(ctx, b: int):
    elems, npar, dt = _i64(), _i32(), _i32()
    _check(ctx, _lib.ddp_get_bucket_info(ctx, b, C.byref(elems), C.byref(npar), C.byref(dt)))
    return elems.value, npar.value, dt.value


def ddp_get_bucket_ptr(ctx, b: int, r: int) -> int:
    p = _vp()
    _check(ctx, _lib.ddp_get_bucket_ptr(ctx, b, r, C.byref(p)))
    return p.value or 0


# The calls made once per parameter go through a small CPython module (plain
# argument passing, a tenth of the interpreter time of a ctypes call); it is
# built together with the library.
import importlib.util as _ilu

_fast_path = os.path.join(_HERE, "_ddp_fastcall.so")
if not os.path.exists(_fast_path):
    raise ImportError(f"{_fast_path} is missing: build it with `python paper_2006_15704_amd/build.py`")
_spec = _ilu.spec_from_file_location("_ddp_fastcall", _fast_path)
_fast = _ilu.module_from_spec(_spec)
_spec.loader.exec_module(_fast)
_fast.bind(C.cast(_lib.ddp_mark_ready, _vp).value, C.cast(_lib.ddp_finalize_backward, _vp).value)
_fast_mark, _fast_finalize = _fast.mark_ready, _fast.finalize_backward


def ddp_mark_ready(ctx, param_id: int) -> None:
    status = _fast_mark(ctx.value, param_id)
    if status < 0:
        _check(ctx, status)


def ddp_mark_ready_local(ctx, param_id: int, used) -> None:
    """used: R flags, non-zero = that replica produced a gradient for the parameter."""
    arr = np.ascontiguousarray([1 if u else 0 for u in used], dtype=np.uint8)
    if arr.size != _replicas.get(ctx.value, arr.size):     # the library reads exactly R bytes
        raise ValueError(f"used has {arr.size} flags, the context has {_replicas[ctx.value]} replicas")
    _check(ctx, _lib.ddp_mark_ready_local(ctx, param_id, _as(arr, C.c_uint8)))


def ddp_get_global_used(ctx, n: int) -> np.ndarray:
    used = np.zeros(n, dtype=np.uint8)
    _check(ctx, _lib.ddp_get_global_used(ctx, _as(used, C.c_uint8)))
    return used


def ddp_mark_ready_many(ctx, ids) -> None:
    arr = _i32_array(ids)
    _check(ctx, _lib.ddp_mark_ready_many(ctx, _as(arr, _i32), len(arr)))


def ddp_finalize_backward(ctx) -> None:
    status = _fast_finalize(ctx.value)
    if status < 0:
        _check(ctx, status)


def ddp_synchronize(ctx) -> None:
    _check(ctx, _lib.ddp_synchronize(ctx))


def ddp_rebuild_buckets(ctx, cap_bytes: int) -> int:
    """New number of buckets; the mapping follows the closed iteration's ready order."""
    return _check(ctx, _lib.ddp_rebuild_buckets(ctx, cap_bytes))


def ddp_get_ready_order(ctx, which: int = 1):
    """Parameters in the order of their ready marks: running (0) or last closed (1) iteration."""
    n = _i32()
    _check(ctx, _lib.ddp_get_ready_order(ctx, which, None, 0, C.byref(n)))
    ids = np.zeros(max(n.value, 1), dtype=np.int32)
    _check(ctx, _lib.ddp_get_ready_order(ctx, which, _as(ids, _i32), n.value, C.byref(n)))
    return [int(x) for x in ids[: n.value]]


def ddp_get_launch_log(ctx, which: int = 1):
    """[(bucket, after_call)] of the running (0) or last closed (1) iteration."""
    n = _i32()
    _check(ctx, _lib.ddp_get_launch_log(ctx, which, None, None, 0, C.byref(n)))
    ids = np.zeros(max(n.value, 1), dtype=np.int32)
    calls = np.zeros(max(n.value, 1), dtype=np.int32)
    _check(ctx, _lib.ddp_get_launch_log(ctx, which, _as(ids, _i32), _as(calls, _i32), n.value, C.byref(n)))
    return [(int(ids[i]), int(calls[i])) for i in range(n.value)]


def ddp_no_sync_accumulate(ctx, micro_grad_ptrs: Sequence[Optional[int]]) -> None:
    arr = _ptr_array(micro_grad_ptrs)
    _check(ctx, _lib.ddp_no_sync_accumulate(ctx, _as(arr, _vp)))


def ddp_get_used_map(ctx, n: int, which: int = 1) -> np.ndarray:
    used = np.zeros(n, dtype=np.uint8)
    _check(ctx, _lib.ddp_get_used_map(ctx, which, _as(used, C.c_uint8)))
    return used


def ddp_synth_backward(ctx, order, delay_ns=None, src_ptrs=None, mark: bool = True) -> None:
    o = _i32_array(order)
    d = None if delay_ns is None else _i64_array(delay_ns)
    s = None if src_ptrs is None else _ptr_array(src_ptrs)
    _check(ctx, _lib.ddp_synth_backward(ctx, _as(o, _i32), len(o),
                                        None if d is None else _as(d, _i64),
                                        None if s is None else _as(s, _vp), 1 if mark else 0))


def ddp_get_kernel_times(ctx, kind: int):
    """(ms[], bucket_id[]) of the timed launches of `kind`."""
    n = _i32()
    _check(ctx, _lib.ddp_get_kernel_times(ctx, kind, None, None, 0, C.byref(n)))
    ms = np.zeros(max(n.value, 1), dtype=np.float32)
    ids = np.zeros(max(n.value, 1), dtype=np.int32)
    _check(ctx, _lib.ddp_get_kernel_times(ctx, kind, _as(ms, C.c_float), _as(ids, _i32), n.value, C.byref(n)))
    return ms[:n.value].copy(), ids[:n.value].copy()


def ddp_sync_static(R: int, device: int, stream: int, numel: Sequence[int], dtype: Sequence[int],
                    grad_ptrs: Sequence[int], cap_bytes: int) -> int:
    """One whole synchronization without a context and without device-memory
    allocation; returns the number of buckets."""
    ne, dt, gp = _i64_array(numel), _i32_array(dtype), _ptr_array(grad_ptrs)
    if len(gp) != R * len(ne):
        raise ValueError(f"grad_ptrs has {len(gp)} entries, expected R*n = {R * len(ne)}")
    return _check(None, _lib.ddp_sync_static(R, device, _vp(stream or None), len(ne), _as(ne, _i64),
                                             _as(dt, _i32), _as(gp, _vp), cap_bytes))
