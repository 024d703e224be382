"""ctypes binding of libdecdec.so: argument marshalling only.

Tensors are passed as raw pointers (`tensor.data_ptr()`); the stream is
torch's current HIP stream unless given.  No step of the hot path is computed
here.  Loading fails loudly if the library has not been built
(`python -m paper_2412_20185_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libdecdec.so")

W_UNIFORM_G128, W_LUT_COL8 = 0, 1
MODE_FUSED, MODE_SERIAL, MODE_TWO_STREAMS = 0, 1, 2
R_FP16, R_INT4_SYM_COL, R_INT2_SYM_COL, R_INT8_SYM_COL = 0, 1, 2, 3
R_FMT_OF_BITS = {16: R_FP16, 4: R_INT4_SYM_COL, 2: R_INT2_SYM_COL, 8: R_INT8_SYM_COL}

EXPORTED_SYMBOLS = (
    "decdec_ws_create", "decdec_ws_destroy", "decdec_sc_buffer_bytes", "decdec_ws_last_selection",
    "decdec_ws_read_selection", "decdec_ws_set_fetch_split", "decdec_ws_set_profiling", "decdec_ws_set_gemv_split", "decdec_ws_set_gemv_waves", "decdec_ws_set_inkernel_accumulate", "decdec_ws_set_separate_select", "decdec_ws_set_mode",
    "decdec_ws_read_profile", "decdec_packed_bytes", "decdec_pack_weights", "decdec_unpack_weights",
    "decdec_pack_residual_int4", "decdec_pack_residual_int", "decdec_select_topk", "decdec_select_bucket", "decdec_gemv", "decdec_gemv_idx", "decdec_gemv_multi",
    "decdec_partial_buffer_bytes", "decdec_ws_read_profile_launches", "decdec_ws_forget_pointer", "decdec_ws_gemv_launch_shape",
    "decdec_ws_pointer_queries", "decdec_gemv_static",
    "decdec_quantize_uniform", "decdec_residual_f32", "decdec_quantize_residual", "decdec_strerror", "decdec_last_hip_error", "decdec_check_pinned", "decdec_check_residual_pointer",
)


class DecdecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().decdec_strerror(status).decode()
        extra = f" (hipError {lib().decdec_last_hip_error()})" if status == -4 else ""
        super().__init__(f"{where}: {msg}{extra} [{status}]")


class Desc(C.Structure):
    _fields_ = [("K", C.c_int32), ("N", C.c_int32), ("wbits", C.c_int32), ("wfmt", C.c_int32), ("rfmt", C.c_int32)]

    def __init__(self, K, N, wbits, wfmt=W_UNIFORM_G128, rfmt=R_FP16):
        super().__init__(int(K), int(N), int(wbits), int(wfmt), int(rfmt))


class Linear(C.Structure):
    """decdec_linear: one weight matrix with its residual and output (for decdec_gemv_multi)."""
    _fields_ = [("desc", C.POINTER(Desc)), ("Wq", C.c_void_p), ("scales", C.c_void_p), ("zeros_or_lut", C.c_void_p),
                ("R_pinned", C.c_void_p), ("R_scales", C.c_void_p), ("y", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it is missing (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(lib_path):
        raise ImportError(f"{lib_path} not found: build it with `python -m paper_2412_20185_amd.build` "
                          "(needs hipcc); there is no CPU fallback")
    L = C.CDLL(lib_path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    dp = C.POINTER(Desc)
    L.decdec_strerror.restype = C.c_char_p
    L.decdec_strerror.argtypes = [C.c_int]
    L.decdec_last_hip_error.restype = C.c_int
    L.decdec_sc_buffer_bytes.restype = sz
    L.decdec_sc_buffer_bytes.argtypes = [i32]
    L.decdec_partial_buffer_bytes.restype = sz
    L.decdec_partial_buffer_bytes.argtypes = [i32]
    L.decdec_ws_read_profile_launches.argtypes = [vp, i32, C.POINTER(C.c_float), i32, C.POINTER(i32)]
    L.decdec_ws_forget_pointer.argtypes = [vp, vp]
    L.decdec_ws_pointer_queries.restype = C.c_int64
    L.decdec_ws_pointer_queries.argtypes = [vp]
    L.decdec_gemv_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    L.decdec_check_pinned.argtypes = [vp]
    L.decdec_check_residual_pointer.argtypes = [vp]
    L.decdec_ws_create.argtypes = [i32, i32, i32, C.POINTER(vp)]
    L.decdec_ws_destroy.argtypes = [vp]
    L.decdec_ws_last_selection.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.decdec_ws_read_selection.argtypes = [vp, i32, vp, vp]
    L.decdec_ws_set_fetch_split.argtypes = [vp, i32]
    L.decdec_ws_set_profiling.argtypes = [vp, i32]
    L.decdec_ws_set_gemv_split.argtypes = [vp, i32]
    L.decdec_ws_set_gemv_waves.argtypes = [vp, i32]
    L.decdec_ws_set_inkernel_accumulate.argtypes = [vp, i32]
    L.decdec_ws_gemv_launch_shape.argtypes = [vp, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    L.decdec_ws_set_separate_select.argtypes = [vp, i32]
    L.decdec_ws_set_mode.argtypes = [vp, i32]
    L.decdec_ws_read_profile.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    L.decdec_packed_bytes.restype = sz
    L.decdec_packed_bytes.argtypes = [dp]
    L.decdec_pack_weights.argtypes = [dp, vp, vp]
    L.decdec_unpack_weights.argtypes = [dp, vp, vp]
    L.decdec_pack_residual_int4.argtypes = [i32, i32, vp, vp]
    L.decdec_pack_residual_int.argtypes = [i32, i32, i32, vp, vp]
    L.decdec_select_topk.argtypes = [vp, i32, i32, vp, vp, vp]
    L.decdec_select_bucket.argtypes = [vp, i32, i32, C.c_float, C.c_float, vp, vp, vp]
    L.decdec_gemv.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    L.decdec_gemv_idx.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    L.decdec_quantize_uniform.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    L.decdec_residual_f32.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    L.decdec_quantize_residual.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    L.decdec_gemv_multi.argtypes = [i32, C.POINTER(Linear), vp, i32, vp, vp]
    _lib = L
    return L


def _check(status: int, where: str):
    if status != 0:
        raise DecdecError(status, where)


def _ptr(t) -> int | None:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return int(t)


def _stream(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def decdec_strerror(status: int) -> str:
    return lib().decdec_strerror(status).decode()


def decdec_sc_buffer_bytes(k: int) -> int:
    return int(lib().decdec_sc_buffer_bytes(k))


def decdec_partial_buffer_bytes(maxN: int) -> int:
    return int(lib().decdec_partial_buffer_bytes(maxN))


STATIC_MAX_N, STATIC_MAX_SELECTED = 32768, 4096


def decdec_check_pinned(t) -> int:
    return int(lib().decdec_check_pinned(_ptr(t)))


def decdec_check_residual_pointer(t) -> int:
    return int(lib().decdec_check_residual_pointer(_ptr(t)))


class Workspace:
    """Owns a decdec_ws (side stream, events, selection and partial buffers)."""

    def __init__(self, maxK: int, maxN: int, maxk: int):
        h = C.c_void_p()
        _check(lib().decdec_ws_create(maxK, maxN, maxk, C.byref(h)), "decdec_ws_create")
        self.handle = h
        self.maxK, self.maxN, self.maxk = maxK, maxN, maxk

    def set_fetch_split(self, row_split: int):
        _check(lib().decdec_ws_set_fetch_split(self.handle, row_split), "decdec_ws_set_fetch_split")

    def set_mode(self, mode: int):
        """MODE_FUSED (default), MODE_SERIAL or MODE_TWO_STREAMS."""
        _check(lib().decdec_ws_set_mode(self.handle, int(mode)), "decdec_ws_set_mode")

    def set_separate_select(self, on: bool):
        _check(lib().decdec_ws_set_separate_select(self.handle, int(on)), "decdec_ws_set_separate_select")

    def set_inkernel_accumulate(self, on: bool):
        _check(lib().decdec_ws_set_inkernel_accumulate(self.handle, int(on)), "decdec_ws_set_inkernel_accumulate")

    def set_gemv_split(self, groups_per_wave: int):
        _check(lib().decdec_ws_set_gemv_split(self.handle, groups_per_wave), "decdec_ws_set_gemv_split")

    def set_gemv_waves(self, waves_per_workgroup: int):
        _check(lib().decdec_ws_set_gemv_waves(self.handle, waves_per_workgroup), "decdec_ws_set_gemv_waves")

    def gemv_launch_shape(self, K: int, N_total: int):
        """(workgroups, threads per workgroup, K-slices) of the base GEMV kernel of a k = 0 call."""
        wg, th, sl = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().decdec_ws_gemv_launch_shape(self.handle, K, N_total, C.byref(wg), C.byref(th), C.byref(sl)),
               "decdec_ws_gemv_launch_shape")
        return wg.value, th.value, sl.value

    def set_profiling(self, capacity: int):
        _check(lib().decdec_ws_set_profiling(self.handle, capacity), "decdec_ws_set_profiling")

    def read_profile(self):
        """Synchronous: {'gemv': (ms_total, launches), 'select': ..., 'fetch': ..., 'accumulate': ...}
        kernel durations since the last read."""
        ms = (C.c_double * 4)()
        n = (C.c_int32 * 4)()
        _check(lib().decdec_ws_read_profile(self.handle, ms, n), "decdec_ws_read_profile")
        return {name: (ms[i], n[i]) for i, name in enumerate(("gemv", "select", "fetch", "accumulate"))}

    KERNEL_CLASSES = ("gemv", "select", "fetch", "accumulate")

    def read_profile_launches(self, kernel_class: str, capacity: int = 1 << 16):
        """Synchronous: the duration (ms) of every timed launch of one kernel class since the last read, in
        call order (this read starts the record over, like read_profile)."""
        buf = (C.c_float * capacity)()
        n = C.c_int32()
        _check(lib().decdec_ws_read_profile_launches(self.handle, self.KERNEL_CLASSES.index(kernel_class), buf,
                                                     capacity, C.byref(n)), "decdec_ws_read_profile_launches")
        return [buf[i] for i in range(n.value)]

    def forget_pointer(self, t=None):
        _check(lib().decdec_ws_forget_pointer(self.handle, _ptr(t)), "decdec_ws_forget_pointer")

    def pointer_queries(self) -> int:
        return int(lib().decdec_ws_pointer_queries(self.handle))

    def last_selection_ptrs(self):
        a, b = C.c_void_p(), C.c_void_p()
        _check(lib().decdec_ws_last_selection(self.handle, C.byref(a), C.byref(b)), "decdec_ws_last_selection")
        return a.value, b.value

    def read_selection(self, k: int):
        """Synchronous: (idx int32 [k], xsel fp16 [k]) of the last decdec_gemv on this workspace."""
        idx = np.empty(k, dtype=np.int32)
        xs = np.empty(k, dtype=np.float16)
        _check(lib().decdec_ws_read_selection(self.handle, k, idx.ctypes.data, xs.ctypes.data),
               "decdec_ws_read_selection")
        return idx, xs

    def close(self):
        if self.handle is not None and self.handle.value:
            lib().decdec_ws_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def decdec_packed_bytes(desc: Desc) -> int:
    return int(lib().decdec_packed_bytes(C.byref(desc)))


def decdec_pack_weights(desc: Desc, codes_KN: np.ndarray) -> np.ndarray:
    """Host: uint8 codes [K][N] -> packed bytes (np.uint8) in the private layout."""
    codes = np.ascontiguousarray(codes_KN, dtype=np.uint8)
    if codes.shape != (desc.K, desc.N):
        raise ValueError("codes shape must be (K, N)")
    out = np.empty(decdec_packed_bytes(desc), dtype=np.uint8)
    _check(lib().decdec_pack_weights(C.byref(desc), codes.ctypes.data, out.ctypes.data), "decdec_pack_weights")
    return out


def decdec_unpack_weights(desc: Desc, packed: np.ndarray) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    if packed.size != decdec_packed_bytes(desc):
        raise ValueError("packed size mismatch")
    out = np.empty((desc.K, desc.N), dtype=np.uint8)
    _check(lib().decdec_unpack_weights(C.byref(desc), packed.ctypes.data, out.ctypes.data), "decdec_unpack_weights")
    return out


def decdec_pack_residual_int4(codes_KN: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes_KN, dtype=np.int8)
    K, N = codes.shape
    out = np.empty((K, N // 2), dtype=np.uint8)
    _check(lib().decdec_pack_residual_int4(K, N, codes.ctypes.data, out.ctypes.data), "decdec_pack_residual_int4")
    return out


def decdec_pack_residual_int(codes_KN: np.ndarray, bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes_KN, dtype=np.int8)
    K, N = codes.shape
    out = np.empty((K, N * bits // 8), dtype=np.uint8)
    _check(lib().decdec_pack_residual_int(K, N, bits, codes.ctypes.data, out.ctypes.data), "decdec_pack_residual_int")
    return out


def decdec_select_topk(x, K: int, k: int, idx_out, xsel_out=None, stream=None):
    _check(lib().decdec_select_topk(_ptr(x), K, k, _ptr(idx_out), _ptr(xsel_out), _stream(stream)),
           "decdec_select_topk")


def decdec_select_bucket(x, K: int, k_chunk: int, b0: float, b15: float, idx_out, xsel_out=None, stream=None):
    _check(lib().decdec_select_bucket(_ptr(x), K, k_chunk, float(b0), float(b15), _ptr(idx_out), _ptr(xsel_out),
                                      _stream(stream)), "decdec_select_bucket")


def decdec_gemv(desc: Desc, x, Wq, scales, zeros_or_lut, R_pinned, R_scales, k: int, y, ws: Workspace, stream=None):
    _check(lib().decdec_gemv(C.byref(desc), _ptr(x), _ptr(Wq), _ptr(scales), _ptr(zeros_or_lut), _ptr(R_pinned),
                             _ptr(R_scales), k, _ptr(y), ws.handle, _stream(stream)), "decdec_gemv")


def decdec_gemv_static(desc: Desc, x, Wq, scales, zeros_or_lut, R_pinned, R_scales, k: int, y, stream=None):
    _check(lib().decdec_gemv_static(C.byref(desc), _ptr(x), _ptr(Wq), _ptr(scales), _ptr(zeros_or_lut),
                                    _ptr(R_pinned), _ptr(R_scales), k, _ptr(y), _stream(stream)),
           "decdec_gemv_static")


def decdec_gemv_idx(desc: Desc, x, Wq, scales, zeros_or_lut, R_pinned, R_scales, k: int, idx, xsel, y,
                    ws: Workspace, stream=None):
    _check(lib().decdec_gemv_idx(C.byref(desc), _ptr(x), _ptr(Wq), _ptr(scales), _ptr(zeros_or_lut), _ptr(R_pinned),
                                 _ptr(R_scales), k, _ptr(idx), _ptr(xsel), _ptr(y), ws.handle, _stream(stream)),
           "decdec_gemv_idx")


def make_linears(items) -> "C.Array":
    """items: iterable of (desc, Wq, scales, zeros_or_lut, R_pinned, R_scales, y) -> ctypes array of decdec_linear.
    Build it once and reuse it: the array keeps the descriptors alive."""
    items = list(items)
    arr = (Linear * len(items))()
    arr._keep = items
    for i, (desc, Wq, scales, zl, R, Rs, y) in enumerate(items):
        arr[i].desc = C.pointer(desc)
        arr[i].Wq, arr[i].scales, arr[i].zeros_or_lut = _ptr(Wq), _ptr(scales), _ptr(zl)
        arr[i].R_pinned, arr[i].R_scales, arr[i].y = _ptr(R), _ptr(Rs), _ptr(y)
    return arr


def decdec_gemv_multi(linears, x, k: int, ws: Workspace, stream=None):
    """linears: array from make_linears() (matrices sharing x)."""
    _check(lib().decdec_gemv_multi(len(linears), linears, _ptr(x), k, ws.handle, _stream(stream)),
           "decdec_gemv_multi")


def decdec_quantize_uniform(desc: Desc, W_f32, Wq_out, scales_out, zeros_out, R_out=None, stream=None):
    _check(lib().decdec_quantize_uniform(C.byref(desc), _ptr(W_f32), _ptr(Wq_out), _ptr(scales_out),
                                         _ptr(zeros_out), _ptr(R_out), _stream(stream)), "decdec_quantize_uniform")


def decdec_residual_f32(desc: Desc, W_f32, Wq, scales, zeros_or_lut, R_f32_out, stream=None):
    _check(lib().decdec_residual_f32(C.byref(desc), _ptr(W_f32), _ptr(Wq), _ptr(scales), _ptr(zeros_or_lut),
                                     _ptr(R_f32_out), _stream(stream)), "decdec_residual_f32")


def decdec_quantize_residual(K: int, N: int, bits: int, R_f32, codes_out, scales_out, stream=None):
    _check(lib().decdec_quantize_residual(K, N, bits, _ptr(R_f32), _ptr(codes_out), _ptr(scales_out),
                                          _stream(stream)), "decdec_quantize_residual")
