"""ctypes binding of liblsr_head.so: argument marshalling only.

Every function here has the name and argument order of its C entry point (include/lsr_head.h) and
does nothing but turn torch tensors into device pointers and pass the current HIP stream.  All of the
head's arithmetic runs in the HIP kernels; there is no fallback: if the library has not been built
or cannot be loaded, importing succeeds but every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

LSR_F32 = 0
LSR_BF16 = 1
LSR_PROFILE_SLOTS = 8
LSR_STATIC_SCRATCH_BYTES = 16 << 20

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblsr_head.so")
_lib = None


class LsrError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lsr_head status {status}: {message}")
        self.status = status


class _BackwardOpts(ctypes.Structure):
    _fields_ = [("grad_dtype", ctypes.c_int32), ("accumulate", ctypes.c_int32)]


class _Desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("S", ctypes.c_int64), ("D", ctypes.c_int64), ("V", ctypes.c_int64),
                ("hw_dtype", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen the in-tree library (build it with paper_2603_25011_amd.build first)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is missing: run `python -m paper_2603_25011_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, fp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(_Desc)
    lib.lsr_head_workspace_bytes.restype = sz
    lib.lsr_head_workspace_bytes.argtypes = [dp, ctypes.c_int]
    lib.lsr_head_forward.restype = ctypes.c_int
    lib.lsr_head_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lsr_head_forward_static.restype = ctypes.c_int
    lib.lsr_head_forward_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.lsr_head_backward.restype = ctypes.c_int
    lib.lsr_head_backward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    op = ctypes.POINTER(_BackwardOpts)
    lib.lsr_head_backward_ex.restype = ctypes.c_int
    lib.lsr_head_backward_ex.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, op, vp, sz, vp]
    lib.lsr_head_backward_ex_workspace_bytes.restype = sz
    lib.lsr_head_backward_ex_workspace_bytes.argtypes = [dp, op]
    lib.lsr_head_forward_profiled.restype = ctypes.c_int
    lib.lsr_head_forward_profiled.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp, fp]
    lib.lsr_head_plan.restype = ctypes.c_int
    lib.lsr_head_plan.argtypes = [dp, ctypes.POINTER(ctypes.c_int32)]
    lib.lsr_mfma_peak_probe.restype = ctypes.c_int
    lib.lsr_mfma_peak_probe.argtypes = [ctypes.c_int64, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.lsr_copy_probe.restype = ctypes.c_int
    lib.lsr_copy_probe.argtypes = [vp, vp, sz, ctypes.c_int, ctypes.POINTER(ctypes.c_double), vp]
    lib.lsr_gather_probe.restype = ctypes.c_int
    lib.lsr_gather_probe.argtypes = [vp, sz, ctypes.c_int, ctypes.c_int, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    lib.lsr_head_backward_profiled.restype = ctypes.c_int
    lib.lsr_head_backward_profiled.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, fp]
    lib.lsr_status_string.restype = ctypes.c_char_p
    lib.lsr_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def lsr_status_string(status: int) -> str:
    return load_library().lsr_status_string(int(status)).decode()


def _desc(B: int, S: int, D: int, V: int, hw_dtype: int) -> _Desc:
    return _Desc(int(B), int(S), int(D), int(V), int(hw_dtype))


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL); raw integers pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int) -> None:
    if rc != 0:
        raise LsrError(rc, lsr_status_string(rc))


def _ws(workspace):
    if workspace is None:
        return None, 0
    if isinstance(workspace, tuple):
        return workspace
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def lsr_head_workspace_bytes(B, S, D, V, hw_dtype, for_backward: bool) -> int:
    d = _desc(B, S, D, V, hw_dtype)
    return int(load_library().lsr_head_workspace_bytes(ctypes.byref(d), 1 if for_backward else 0))


def lsr_head_forward(B, S, D, V, hw_dtype, H, W, bias, mask, Y, I, workspace, stream=None) -> None:
    d = _desc(B, S, D, V, hw_dtype)
    wp, wb = _ws(workspace)
    _check(load_library().lsr_head_forward(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(bias), _ptr(mask), _ptr(Y),
                                           _ptr(I), wp, wb, _stream(stream)))


def lsr_head_forward_static(B, S, D, V, hw_dtype, H, W, bias, mask, Y, I, stream=None) -> None:
    d = _desc(B, S, D, V, hw_dtype)
    _check(load_library().lsr_head_forward_static(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(bias), _ptr(mask), _ptr(Y),
                                                  _ptr(I), _stream(stream)))


def lsr_head_backward(B, S, D, V, hw_dtype, H, W, dY, Y, I, dH, dW, db, workspace, stream=None) -> None:
    d = _desc(B, S, D, V, hw_dtype)
    wp, wb = _ws(workspace)
    _check(load_library().lsr_head_backward(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(dY), _ptr(Y), _ptr(I),
                                            _ptr(dH), _ptr(dW), _ptr(db), wp, wb, _stream(stream)))


def lsr_head_backward_ex_workspace_bytes(B, S, D, V, hw_dtype, grad_dtype=LSR_F32, accumulate=False) -> int:
    d = _desc(B, S, D, V, hw_dtype)
    o = _BackwardOpts(int(grad_dtype), 1 if accumulate else 0)
    return int(load_library().lsr_head_backward_ex_workspace_bytes(ctypes.byref(d), ctypes.byref(o)))


def lsr_head_backward_ex(B, S, D, V, hw_dtype, H, W, dY, Y, I, dH, dW, db, grad_dtype, accumulate, workspace,
                         stream=None) -> None:
    d = _desc(B, S, D, V, hw_dtype)
    o = _BackwardOpts(int(grad_dtype), 1 if accumulate else 0)
    wp, wb = _ws(workspace)
    _check(load_library().lsr_head_backward_ex(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(dY), _ptr(Y), _ptr(I),
                                               _ptr(dH), _ptr(dW), _ptr(db), ctypes.byref(o), wp, wb, _stream(stream)))


def lsr_head_forward_profiled(B, S, D, V, hw_dtype, H, W, bias, mask, Y, I, workspace, stream=None):
    d = _desc(B, S, D, V, hw_dtype)
    wp, wb = _ws(workspace)
    ms = (ctypes.c_float * LSR_PROFILE_SLOTS)()
    _check(load_library().lsr_head_forward_profiled(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(bias), _ptr(mask),
                                                    _ptr(Y), _ptr(I), wp, wb, _stream(stream), ms))
    return list(ms)


LSR_PLAN_FIELDS = ("fwd_tiles_per_chunk", "sort_segments", "sort_segment_len", "sort_places_through_lds",
                   "dh_chunks", "dh_chunk_len", "dh_buckets_per_wave", "dw_tile_rows", "dw_sequences_per_launch",
                   "fwd_chunks", "fwd_segment_rows", "fwd_resident_workgroups", "dh_slices_owned_by_xcd",
                   "dw_lds_tile_passes")


def lsr_head_plan(B, S, D, V, hw_dtype):
    """The host's launch plan for a shape, as a dict (no device needed)."""
    d = _desc(B, S, D, V, hw_dtype)
    out = (ctypes.c_int32 * len(LSR_PLAN_FIELDS))()
    _check(load_library().lsr_head_plan(ctypes.byref(d), out))
    return dict(zip(LSR_PLAN_FIELDS, (int(x) for x in out)))


def lsr_mfma_peak_probe(iters, launches, sink, stream=None):
    """Dense bf16 TFLOP/s of register-only MFMAs on the current device (measurement aid)."""
    out = ctypes.c_double(0.0)
    _check(load_library().lsr_mfma_peak_probe(int(iters), int(launches), _ptr(sink), ctypes.byref(out), _stream(stream)))
    return out.value


def lsr_copy_probe(dst, src, nbytes, launches=3, stream=None):
    """GB/s (read + written) of a plain device copy of nbytes (measurement aid)."""
    out = ctypes.c_double(0.0)
    _check(load_library().lsr_copy_probe(_ptr(dst), _ptr(src), int(nbytes), int(launches), ctypes.byref(out), _stream(stream)))
    return out.value


def lsr_gather_probe(table, window_bytes, steps, out, launches=3, stream=None):
    """GB/s of 128-byte row pieces gathered at random rows of a window of the table (measurement aid)."""
    rate = ctypes.c_double(0.0)
    _check(load_library().lsr_gather_probe(_ptr(table), int(window_bytes), int(steps), int(launches), _ptr(out),
                                           out.numel() * out.element_size(), ctypes.byref(rate), _stream(stream)))
    return rate.value


def lsr_head_backward_profiled(B, S, D, V, hw_dtype, H, W, dY, Y, I, dH, dW, db, workspace, stream=None):
    d = _desc(B, S, D, V, hw_dtype)
    wp, wb = _ws(workspace)
    ms = (ctypes.c_float * LSR_PROFILE_SLOTS)()
    _check(load_library().lsr_head_backward_profiled(ctypes.byref(d), _ptr(H), _ptr(W), _ptr(dY), _ptr(Y), _ptr(I),
                                                     _ptr(dH), _ptr(dW), _ptr(db), wp, wb, _stream(stream), ms))
    return list(ms)
