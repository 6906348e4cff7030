"""Thin Python binding of the PCONV HIP library (argument marshalling only).

Every step of the path - analysis, reorder, compact storage (pconv_pack) and the sparse
convolution (pconv_conv2d) - runs inside libpconv.so; PyTorch appears only as the owner of
device memory and streams.  There is no CPU fallback: if the library is missing or no GPU is
present, calls fail loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import _build

F32, BF16 = 0, 1
NCHW, NHWC = 0, 1
OK, INVALID_ARG, OOM, HIP_ERROR, UNSUPPORTED = 0, -1, -2, -3, -4
MAX_PATTERNS = 16

_DTYPE = {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}
_LAYOUT = {"nchw": NCHW, "nhwc": NHWC, NCHW: NCHW, NHWC: NHWC}


class PconvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pconv status {status}: {message}")
        self.status = status


class pconv_info(C.Structure):
    _fields_ = [("c_out", C.c_int32), ("c_in", C.c_int32), ("num_patterns", C.c_int32),
                ("weight_dtype", C.c_int32), ("kept_kernels", C.c_int64), ("nnz", C.c_int64),
                ("device_bytes", C.c_int64), ("fast_path", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """Load libpconv.so (built in-tree by __graft_entry__.build(); built here only if absent)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        _build.build()
    L = C.CDLL(path)
    vp, ip = C.c_void_p, C.c_int
    L.pconv_pack.restype = ip
    L.pconv_pack.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, C.POINTER(vp)]
    L.pconv_project.restype = ip
    L.pconv_project.argtypes = [vp, vp, ip, ip, ip, C.c_int64, vp, vp]
    L.pconv_debug_pack_host.restype = ip
    L.pconv_debug_pack_host.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, C.POINTER(vp)]
    L.pconv_conv2d.restype = ip
    L.pconv_conv2d.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, ip, vp]
    L.pconv_conv2d_static.restype = ip
    L.pconv_conv2d_static.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, ip, vp]
    L.pconv_conv2d_pool2x2.restype = ip
    L.pconv_conv2d_pool2x2.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, vp]
    L.pconv_free.restype = None
    L.pconv_free.argtypes = [vp]
    L.pconv_maxpool2x2.restype = ip
    L.pconv_maxpool2x2.argtypes = [vp, vp, ip, ip, ip, ip, ip, ip, vp]
    L.pconv_get_info.restype = ip
    L.pconv_get_info.argtypes = [vp, C.POINTER(pconv_info)]
    L.pconv_debug_export.restype = ip
    L.pconv_debug_export.argtypes = [vp, vp, vp, vp, vp, vp]
    L.pconv_debug_export_blocks.restype = ip
    L.pconv_debug_export_blocks.argtypes = [vp, vp, vp]
    L.pconv_debug_unpack.restype = ip
    L.pconv_debug_unpack.argtypes = [vp, vp]
    L.pconv_set_kernel_policy.restype = ip
    L.pconv_set_kernel_policy.argtypes = [ip]
    L.pconv_debug_set_tiling.restype = ip
    L.pconv_debug_set_tiling.argtypes = [ip, ip, ip]
    L.pconv_debug_set_spin_limit.restype = ip
    L.pconv_debug_set_spin_limit.argtypes = [ip]
    L.pconv_get_async_error.restype = ip
    L.pconv_get_async_error.argtypes = [vp]
    L.pconv_pool2x2_fusion.restype = ip
    L.pconv_pool2x2_fusion.argtypes = [vp, ip, ip, ip, ip, ip]
    L.pconv_debug_measure_fma_peak.restype = ip
    L.pconv_debug_measure_fma_peak.argtypes = [C.POINTER(C.c_double)]
    L.pconv_last_error.restype = C.c_char_p
    L.pconv_last_error.argtypes = []
    _lib = L
    return L


EXPORTED_SYMBOLS = ["pconv_project", "pconv_pack", "pconv_conv2d", "pconv_conv2d_static", "pconv_conv2d_pool2x2", "pconv_free", "pconv_maxpool2x2",
                    "pconv_get_info", "pconv_debug_export", "pconv_debug_export_blocks", "pconv_debug_pack_host",
                    "pconv_debug_unpack",
                    "pconv_set_kernel_policy", "pconv_debug_set_tiling", "pconv_debug_set_spin_limit",
                    "pconv_get_async_error", "pconv_pool2x2_fusion", "pconv_debug_measure_fma_peak",
                    "pconv_last_error"]


def _check(rc: int):
    if rc != OK:
        raise PconvError(rc, lib().pconv_last_error().decode())


def _np(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


class Handle:
    """Owns one pconv_handle*; free() or garbage collection releases it."""

    def __init__(self, ptr: int, c_out: int, c_in: int, dtype: int):
        self.ptr, self.c_out, self.c_in, self.dtype = ptr, c_out, c_in, dtype

    def info(self) -> pconv_info:
        out = pconv_info()
        _check(lib().pconv_get_info(self.ptr, C.byref(out)))
        return out

    def free(self):
        if self.ptr:
            lib().pconv_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pconv_pack(w_dense, pattern_id, conn, table, weight_dtype="f32", host_only=False) -> Handle:
    """Host arrays -> packed device handle (see include/pconv.h).

    host_only=True calls pconv_debug_pack_host instead (no GPU needed, no device data)."""
    w = _np(w_dense, np.float32)
    pid = _np(pattern_id, np.uint8)
    cn = _np(conn, np.uint8)
    tb = _np(table, np.uint16)
    if w.ndim != 4 or w.shape[2:] != (3, 3) or pid.shape != w.shape[:2] or cn.shape != w.shape[:2]:
        raise ValueError("expected w [F][C][3][3] and pattern_id/conn [F][C]")
    out = C.c_void_p()
    fn = lib().pconv_debug_pack_host if host_only else lib().pconv_pack
    rc = fn(w.ctypes.data, pid.ctypes.data, cn.ctypes.data, tb.ctypes.data,
            int(tb.size), int(w.shape[0]), int(w.shape[1]), _DTYPE[weight_dtype], C.byref(out))
    _check(rc)
    return Handle(out.value, int(w.shape[0]), int(w.shape[1]), _DTYPE[weight_dtype])


def pconv_project(w_dense, table, keep_kernels: int):
    """Dense weights [F][C][3][3] -> (pattern_id [F][C] uint8, conn [F][C] uint8); see include/pconv.h."""
    w = _np(w_dense, np.float32)
    tb = _np(table, np.uint16)
    if w.ndim != 4 or w.shape[2:] != (3, 3):
        raise ValueError("expected w [F][C][3][3]")
    pid = np.empty(w.shape[:2], np.uint8)
    conn = np.empty(w.shape[:2], np.uint8)
    _check(lib().pconv_project(w.ctypes.data, tb.ctypes.data, int(tb.size), int(w.shape[0]), int(w.shape[1]),
                               int(keep_kernels), pid.ctypes.data, conn.ctypes.data))
    return pid, conn


def pconv_conv2d(handle: Handle, x_ptr: int, y_ptr: int, bias_ptr, n: int, h_in: int, w_in: int,
                 stride: int = 1, pad: int = 1, layout=NCHW, act_dtype=F32, fuse_relu: bool = False,
                 stream: int = 0):
    """Raw-pointer call, one to one with the C entry point."""
    _check(lib().pconv_conv2d(handle.ptr, x_ptr, y_ptr, bias_ptr or None, n, h_in, w_in, stride, pad,
                              _LAYOUT[layout], _DTYPE[act_dtype], int(bool(fuse_relu)),
                              stream or None))


def pconv_conv2d_static(handle: Handle, x_ptr: int, y_ptr: int, bias_ptr, n: int, h_in: int, w_in: int,
                        stride: int = 1, pad: int = 1, layout=NCHW, act_dtype=F32, fuse_relu: bool = False,
                        stream: int = 0):
    """Raw-pointer call, one to one with the C entry point."""
    _check(lib().pconv_conv2d_static(handle.ptr, x_ptr, y_ptr, bias_ptr or None, n, h_in, w_in, stride, pad,
                                     _LAYOUT[layout], _DTYPE[act_dtype], int(bool(fuse_relu)),
                                     stream or None))


def pconv_conv2d_pool2x2(handle: Handle, x_ptr: int, y_ptr: int, bias_ptr, n: int, h_in: int, w_in: int,
                         layout=NCHW, act_dtype=F32, fuse_relu: bool = False, stream: int = 0):
    """Raw-pointer call, one to one with the C entry point."""
    _check(lib().pconv_conv2d_pool2x2(handle.ptr, x_ptr, y_ptr, bias_ptr or None, n, h_in, w_in,
                                      _LAYOUT[layout], _DTYPE[act_dtype], int(bool(fuse_relu)),
                                      stream or None))


def pconv_free(handle: Handle):
    handle.free()


def pconv_maxpool2x2(x_ptr: int, y_ptr: int, n: int, c: int, h: int, w: int, layout=NCHW,
                     dtype=F32, stream: int = 0):
    _check(lib().pconv_maxpool2x2(x_ptr, y_ptr, n, c, h, w, _LAYOUT[layout], _DTYPE[dtype],
                                  stream or None))


def pconv_set_kernel_policy(policy: int):
    """0 automatic, 1 generic gather kernel, 2 register-tiled vector kernel, 3 matrix-core kernel (bf16)."""
    _check(lib().pconv_set_kernel_policy(int(policy)))


def pconv_debug_set_tiling(waves: int = 0, ks_log2: int = -1, split_units: int = -1):
    _check(lib().pconv_debug_set_tiling(int(waves), int(ks_log2), int(split_units)))


def pconv_pool2x2_fusion(handle: Handle, n: int, h_in: int, w_in: int, layout=NCHW, act_dtype=F32) -> int:
    """0 = the fused call is not supported, 1 = supported but not recommended, 2 = recommended."""
    rc = lib().pconv_pool2x2_fusion(handle.ptr, n, h_in, w_in, _LAYOUT[layout], _DTYPE[act_dtype])
    if rc < 0:
        _check(rc)
    return rc


def pconv_debug_measure_fma_peak() -> float:
    out = C.c_double()
    _check(lib().pconv_debug_measure_fma_peak(C.byref(out)))
    return out.value


def pconv_debug_set_spin_limit(limit: int = 0):
    _check(lib().pconv_debug_set_spin_limit(int(limit)))


def pconv_get_async_error(handle: Handle):
    """Raises PconvError(HIP_ERROR) once if a kernel on this handle gave up a bounded wait."""
    _check(lib().pconv_get_async_error(handle.ptr))


def pconv_debug_export_blocks(handle: Handle):
    """(slot_filter [B][4] int32, records [B][J] uint32): see include/pconv.h."""
    info = handle.info()
    b, j = -(-info.c_out // 4), -(-info.c_in // 8)
    slot_filter = np.empty((b, 4), np.int32); records = np.empty((b, j), np.uint32)
    _check(lib().pconv_debug_export_blocks(handle.ptr, slot_filter.ctypes.data, records.ctypes.data))
    return slot_filter, records


def pconv_debug_export(handle: Handle) -> dict:
    info = handle.info()
    f, p = info.c_out, info.num_patterns
    perm = np.empty(f, np.uint16); row_ptr = np.empty(f + 1, np.uint32)
    pat_cnt = np.empty((f, p), np.uint16); cin = np.empty(info.kept_kernels, np.uint16)
    vals = np.empty(info.nnz, np.float32 if info.weight_dtype == F32 else np.uint16)
    _check(lib().pconv_debug_export(handle.ptr, perm.ctypes.data, row_ptr.ctypes.data,
                                    pat_cnt.ctypes.data, cin.ctypes.data, vals.ctypes.data))
    return dict(perm=perm, row_ptr=row_ptr, pat_cnt=pat_cnt, cin=cin, vals=vals)


def pconv_debug_unpack(handle: Handle) -> np.ndarray:
    w = np.empty((handle.c_out, handle.c_in, 3, 3), np.float32)
    _check(lib().pconv_debug_unpack(handle.ptr, w.ctypes.data))
    return w


# ---- torch conveniences (device memory + streams only) ---------------------------------

def _torch_dtype(dtype):
    import torch
    return torch.float32 if _DTYPE[dtype] == F32 else torch.bfloat16


def conv2d(handle: Handle, x, bias=None, stride: int = 1, relu: bool = False, layout="nchw",
           out=None):
    """x: CUDA tensor (NCHW or NHWC contiguous). Returns y on the same device/stream."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous CUDA tensor")
    lay = _LAYOUT[layout]
    if lay == NCHW:
        n, c, h, w = x.shape
    else:
        n, h, w, c = x.shape
    if c != handle.c_in:
        raise ValueError("channel count does not match the handle")
    if x.dtype != _torch_dtype(handle.dtype):
        raise ValueError("activation dtype does not match the handle")
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    shape = (n, handle.c_out, ho, wo) if lay == NCHW else (n, ho, wo, handle.c_out)
    y = out if out is not None else torch.empty(shape, dtype=x.dtype, device=x.device)
    if bias is not None and (bias.dtype != torch.float32 or not bias.is_cuda):
        raise ValueError("bias must be a float32 CUDA tensor")
    stream = torch.cuda.current_stream(x.device).cuda_stream
    pconv_conv2d(handle, x.data_ptr(), y.data_ptr(), bias.data_ptr() if bias is not None else 0,
                 n, h, w, stride, 1, lay, handle.dtype, relu, stream)
    return y


def conv2d_pool2x2(handle: Handle, x, bias=None, relu: bool = False, out=None):
    """x: contiguous fp32 NCHW CUDA tensor.  Returns maxpool2x2(conv2d(x)) without the intermediate."""
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous CUDA tensor")
    n, c, h, w = x.shape
    if c != handle.c_in:
        raise ValueError("channel count does not match the handle")
    if x.dtype != _torch_dtype(handle.dtype):
        raise ValueError("activation dtype does not match the handle")
    y = out if out is not None else torch.empty((n, handle.c_out, h // 2, w // 2), dtype=x.dtype, device=x.device)
    if bias is not None and (bias.dtype != torch.float32 or not bias.is_cuda):
        raise ValueError("bias must be a float32 CUDA tensor")
    stream = torch.cuda.current_stream(x.device).cuda_stream
    pconv_conv2d_pool2x2(handle, x.data_ptr(), y.data_ptr(), bias.data_ptr() if bias is not None else 0,
                         n, h, w, NCHW, handle.dtype, relu, stream)
    return y


def maxpool2x2(x, layout="nchw"):
    import torch
    lay = _LAYOUT[layout]
    if lay == NCHW:
        n, c, h, w = x.shape
        shape = (n, c, h // 2, w // 2)
    else:
        n, h, w, c = x.shape
        shape = (n, h // 2, w // 2, c)
    y = torch.empty(shape, dtype=x.dtype, device=x.device)
    dt = F32 if x.dtype == torch.float32 else BF16
    pconv_maxpool2x2(x.data_ptr(), y.data_ptr(), n, c, h, w, lay, dt,
                     torch.cuda.current_stream(x.device).cuda_stream)
    return y
