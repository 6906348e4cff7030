"""ctypes binding of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never touches the GPU and shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

F32, BF16 = 0, 1
NCHW, NHWC = 0, 1
_LAYOUT = {"nchw": NCHW, "nhwc": NHWC}
_DTYPE = {"f32": F32, "bf16": BF16}

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        _lib.orc_bf16_bits.restype = C.c_uint16
        _lib.orc_bf16_bits.argtypes = [C.c_float]
        _lib.orc_bf16_value.restype = C.c_float
        _lib.orc_bf16_value.argtypes = [C.c_float]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def bf16_bits(v: float) -> int:
    return int(lib().orc_bf16_bits(C.c_float(v)))


def masked_weights(w, pattern_id, conn, table, wdtype="f32") -> np.ndarray:
    """W~ = W (.) P (.) conn as float64 [C_out][C_in][3][3]."""
    w = _c(w, np.float32); pid = _c(pattern_id, np.uint8); cn = _c(conn, np.uint8)
    tb = _c(table, np.uint16)
    f, c = pid.shape
    wt = np.empty((f, c, 3, 3), dtype=np.float64)
    lib().orc_masked_weights(_p(w), _p(pid), _p(cn), _p(tb), C.c_int(f), C.c_int(c),
                             C.c_int(_DTYPE[wdtype]), _p(wt))
    return wt


def _dims(x, layout):
    if layout == "nchw":
        n, c, h, w = x.shape
    else:
        n, h, w, c = x.shape
    return n, c, h, w


def conv2d(x, wt, bias=None, stride=1, pad=1, relu=False, layout="nchw"):
    """Full output (y, S) in float64, same layout as x."""
    x = _c(x, np.float32); wt = _c(wt, np.float64)
    n, c, h, w = _dims(x, layout)
    f = wt.shape[0]
    assert wt.shape == (f, c, 3, 3)
    ho = (h + 2 * pad - 3) // stride + 1
    wo = (w + 2 * pad - 3) // stride + 1
    shape = (n, f, ho, wo) if layout == "nchw" else (n, ho, wo, f)
    y = np.empty(shape, dtype=np.float64); s = np.empty(shape, dtype=np.float64)
    b = _c(bias, np.float32) if bias is not None else None
    lib().orc_conv2d(_p(x), C.c_int(_LAYOUT[layout]), C.c_int(n), C.c_int(c), C.c_int(h),
                     C.c_int(w), _p(wt), C.c_int(f), _p(b), C.c_int(stride), C.c_int(pad),
                     C.c_int(int(relu)), _p(y), _p(s))
    return y, s


def conv2d_points(x, wt, pts, bias=None, stride=1, pad=1, relu=False, layout="nchw"):
    """(y, S) at output points pts[i] = (n, f, y, x)."""
    x = _c(x, np.float32); wt = _c(wt, np.float64)
    pts = _c(pts, np.int32).reshape(-1, 4)
    n, c, h, w = _dims(x, layout)
    f = wt.shape[0]
    y = np.empty(len(pts), dtype=np.float64); s = np.empty(len(pts), dtype=np.float64)
    b = _c(bias, np.float32) if bias is not None else None
    lib().orc_conv2d_points(_p(x), C.c_int(_LAYOUT[layout]), C.c_int(n), C.c_int(c),
                            C.c_int(h), C.c_int(w), _p(wt), C.c_int(f), _p(b),
                            C.c_int(stride), C.c_int(pad), C.c_int(int(relu)),
                            _p(pts), C.c_int64(len(pts)), _p(y), _p(s))
    return y, s


def maxpool2x2(x, layout="nchw"):
    x = _c(x, np.float32)
    n, c, h, w = _dims(x, layout)
    shape = (n, c, h // 2, w // 2) if layout == "nchw" else (n, h // 2, w // 2, c)
    y = np.empty(shape, dtype=np.float32)
    lib().orc_maxpool2x2(_p(x), C.c_int(_LAYOUT[layout]), C.c_int(n), C.c_int(c),
                         C.c_int(h), C.c_int(w), _p(y))
    return y


def pack(w, pattern_id, conn, table, wdtype="f32"):
    """Canonical filter-kernel-reorder layout: dict(perm,row_ptr,pat_cnt,cin,vals)."""
    w = _c(w, np.float32); pid = _c(pattern_id, np.uint8); cn = _c(conn, np.uint8)
    tb = _c(table, np.uint16)
    f, c = pid.shape
    p = len(tb)
    k = C.c_int64(); nnz = C.c_int64()
    lib().orc_pack_sizes(_p(pid), _p(cn), _p(tb), C.c_int(f), C.c_int(c),
                         C.byref(k), C.byref(nnz))
    perm = np.empty(f, np.uint16); row_ptr = np.empty(f + 1, np.uint32)
    pat_cnt = np.empty((f, p), np.uint16); cin = np.empty(k.value, np.uint16)
    vals = np.empty(nnz.value, np.float32 if wdtype == "f32" else np.uint16)
    lib().orc_pack(_p(w), _p(pid), _p(cn), _p(tb), C.c_int(p), C.c_int(f), C.c_int(c),
                   C.c_int(_DTYPE[wdtype]), _p(perm), _p(row_ptr), _p(pat_cnt), _p(cin), _p(vals))
    return dict(perm=perm, row_ptr=row_ptr, pat_cnt=pat_cnt, cin=cin, vals=vals)


def unpack(packed, table, c_in, wdtype="f32"):
    tb = _c(table, np.uint16)
    f = len(packed["perm"])
    w = np.empty((f, c_in, 3, 3), np.float32)
    lib().orc_unpack(_p(packed["perm"]), _p(packed["row_ptr"]), _p(packed["pat_cnt"]),
                     _p(packed["cin"]), _p(packed["vals"]), _p(tb), C.c_int(len(tb)),
                     C.c_int(f), C.c_int(c_in), C.c_int(_DTYPE[wdtype]), _p(w))
    return w


def project(w, table, keep: int):
    """Euclidean projection of dense weights [F][C][3][3] onto (pattern table, `keep` kernels):
    returns (pattern_id [F][C] uint8, conn [F][C] uint8).  See pconv_project_oracle.c."""
    w = _c(w, np.float32)
    tb = _c(table, np.uint16)
    f, c = w.shape[:2]
    pid = np.zeros((f, c), np.uint8)
    conn = np.zeros((f, c), np.uint8)
    fn = lib().orc_project
    fn.restype = None
    fn.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_long, C.c_void_p, C.c_void_p]
    fn(_p(w), _p(tb), int(tb.size), int(f), int(c), int(keep), _p(pid), _p(conn))
    return pid, conn
