"""ctypes binding of libmi355conv.so: same names as include/mi355conv.h.

Argument marshalling only.  PyTorch-ROCm supplies device memory and streams; every
step of the convolution runs in the library's HIP kernels.  There is no fallback:
if the shared library is missing, importing it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmi355conv.so")

ALGO_AUTO, ALGO_IGEMM, ALGO_WINOGRAD, ALGO_WINOGRAD4, ALGO_FFT = 0, 1, 2, 3, 4
OP_FWD, OP_BWD_DATA, OP_BWD_WEIGHT = 0, 1, 2

STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("conv2d_output_dims", "conv2d_pick_algo", "conv2d_workspace_bytes", "conv2d_fwd", "conv2d_fwd_static",
           "conv2d_fwd_relu", "conv2d_fwd_relu_pool2",
           "conv2d_fwd_1x1_group", "conv2d_bwd_data", "conv2d_bwd_weight", "conv2d_status_string", "conv2d_version",
           "apply_mul_add", "conv2d_profile_begin", "conv2d_profile_end", "conv2d_profile_record",
           "conv2d_profile_kernel_name", "conv2d_probe_mfma_f32", "conv2d_probe_copy")


class conv2d_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "C", "H", "W", "K", "R", "S",
                                         "stride_h", "stride_w", "pad_h", "pad_w")]


class Conv2dError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def load() -> C.CDLL:
    """Load the in-tree shared library (built by paper_1606_04884_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libmi355conv.so is not built: run `python -m paper_1606_04884_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    dp = C.POINTER(conv2d_desc)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.conv2d_output_dims.argtypes = [dp, i32p, i32p]
    lib.conv2d_output_dims.restype = C.c_int
    lib.conv2d_pick_algo.argtypes = [dp, C.c_int]
    lib.conv2d_pick_algo.restype = C.c_int
    lib.conv2d_workspace_bytes.argtypes = [dp, C.c_int, C.c_int]
    lib.conv2d_workspace_bytes.restype = C.c_size_t
    lib.conv2d_fwd.argtypes = [dp, vp, vp, vp, vp, vp, C.c_size_t, C.c_int, vp]
    lib.conv2d_fwd.restype = C.c_int
    lib.conv2d_fwd_static.argtypes = [dp, vp, vp, vp, vp, C.c_int, vp]
    lib.conv2d_fwd_static.restype = C.c_int
    lib.conv2d_fwd_relu.argtypes = lib.conv2d_fwd.argtypes
    lib.conv2d_fwd_relu.restype = C.c_int
    lib.conv2d_fwd_relu_pool2.argtypes = [dp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.conv2d_fwd_relu_pool2.restype = C.c_int
    lib.conv2d_fwd_1x1_group.argtypes = [dp, vp, C.c_int32, i32p, C.POINTER(vp), C.POINTER(vp),
                                         C.POINTER(vp), vp, C.c_size_t, vp]
    lib.conv2d_fwd_1x1_group.restype = C.c_int
    lib.conv2d_bwd_data.argtypes = [dp, vp, vp, vp, vp, C.c_size_t, C.c_int, vp]
    lib.conv2d_bwd_data.restype = C.c_int
    lib.conv2d_bwd_weight.argtypes = [dp, vp, vp, vp, vp, C.c_float, C.c_int, vp, C.c_size_t,
                                      C.c_int, vp]
    lib.conv2d_bwd_weight.restype = C.c_int
    lib.apply_mul_add.argtypes = [vp, vp, C.c_int64, C.c_float, C.c_float, vp]
    lib.apply_mul_add.restype = C.c_int
    lib.conv2d_profile_begin.argtypes = [C.c_int]
    lib.conv2d_profile_begin.restype = C.c_int
    lib.conv2d_profile_end.argtypes = []
    lib.conv2d_profile_end.restype = C.c_int
    lib.conv2d_profile_record.argtypes = [C.c_int, i32p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                          C.POINTER(C.c_float)]
    lib.conv2d_profile_record.restype = C.c_int
    lib.conv2d_profile_kernel_name.argtypes = [C.c_int]
    lib.conv2d_profile_kernel_name.restype = C.c_char_p
    lib.conv2d_probe_mfma_f32.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), vp]
    lib.conv2d_probe_mfma_f32.restype = C.c_int
    lib.conv2d_probe_copy.argtypes = [vp, vp, C.c_int64, vp]
    lib.conv2d_probe_copy.restype = C.c_int
    lib.conv2d_status_string.argtypes = [C.c_int]
    lib.conv2d_status_string.restype = C.c_char_p
    lib.conv2d_version.argtypes = []
    lib.conv2d_version.restype = C.c_char_p
    _lib = lib
    return lib


def make_desc(geom: Sequence[int]) -> conv2d_desc:
    """geom = (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w)."""
    g = [int(v) for v in geom]
    if len(g) != 11:
        raise ValueError("geom must have 11 entries")
    return conv2d_desc(*g)


def _desc(d) -> conv2d_desc:
    return d if isinstance(d, conv2d_desc) else make_desc(d)


def status_string(status: int) -> str:
    return load().conv2d_status_string(int(status)).decode()


def conv2d_status_string(status: int) -> str:
    return status_string(status)


def conv2d_version() -> str:
    return load().conv2d_version().decode()


def conv2d_output_dims(d) -> Tuple[int, int]:
    P, Q = C.c_int32(), C.c_int32()
    rc = load().conv2d_output_dims(C.byref(_desc(d)), C.byref(P), C.byref(Q))
    if rc:
        raise Conv2dError(rc, "conv2d_output_dims")
    return P.value, Q.value


def conv2d_pick_algo(d, op: int) -> int:
    rc = load().conv2d_pick_algo(C.byref(_desc(d)), int(op))
    if rc < 0:
        raise Conv2dError(rc, "conv2d_pick_algo")
    return rc


def conv2d_workspace_bytes(d, op: int, algo: int = ALGO_AUTO) -> int:
    return int(load().conv2d_workspace_bytes(C.byref(_desc(d)), int(op), int(algo)))


# ---- tensor marshalling ----------------------------------------------------
def _ptr(t, shape, name: str) -> int:
    import torch
    if t is None:
        return 0
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous float32" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return t.data_ptr()


def _stream(stream) -> int:
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def alloc_workspace(nbytes: int, device="cuda"):
    """A device byte buffer of at least nbytes (torch only provides the memory)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _ws(ws, need: int, stream=None):
    """Caller's workspace, or a temporary one.  A temporary is released when the Python call
    returns while the kernels are only enqueued: it is recorded on the stream they run on, so
    that torch's allocator does not hand the block out again before they have finished."""
    if ws is None:
        import torch
        ws = alloc_workspace(need)
        s = _stream(stream)
        if s != torch.cuda.current_stream().cuda_stream:
            ws.record_stream(torch.cuda.ExternalStream(s))
    return ws, ws.data_ptr(), ws.numel() * ws.element_size()


def conv2d_fwd(d, x, w, bias, y, ws=None, algo: int = ALGO_AUTO, stream=None) -> None:
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_FWD, algo), stream)
    rc = load().conv2d_fwd(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"),
                           _ptr(w, (dd.K, dd.C, dd.R, dd.S), "w"), _ptr(bias, (dd.K,), "bias"),
                           _ptr(y, (dd.N, dd.K, P, Q), "y"), wptr, wbytes, int(algo),
                           _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_fwd")


def conv2d_fwd_static(d, x, w, bias, y, algo: int = ALGO_AUTO, stream=None) -> None:
    """conv2d_fwd with the library's own static scratch area as workspace: nothing is
    allocated here or in the library."""
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    rc = load().conv2d_fwd_static(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"),
                                  _ptr(w, (dd.K, dd.C, dd.R, dd.S), "w"), _ptr(bias, (dd.K,), "bias"),
                                  _ptr(y, (dd.N, dd.K, P, Q), "y"), int(algo), _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_fwd_static")


def conv2d_fwd_relu(d, x, w, bias, y, ws=None, algo: int = ALGO_AUTO, stream=None) -> None:
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_FWD, algo), stream)
    rc = load().conv2d_fwd_relu(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"),
                                _ptr(w, (dd.K, dd.C, dd.R, dd.S), "w"), _ptr(bias, (dd.K,), "bias"),
                                _ptr(y, (dd.N, dd.K, P, Q), "y"), wptr, wbytes, int(algo),
                                _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_fwd_relu")


def conv2d_fwd_relu_pool2(d, x, w, bias, y_pooled, ws=None, stream=None) -> None:
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_FWD, ALGO_WINOGRAD), stream)
    rc = load().conv2d_fwd_relu_pool2(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"),
                                      _ptr(w, (dd.K, dd.C, dd.R, dd.S), "w"), _ptr(bias, (dd.K,), "bias"),
                                      _ptr(y_pooled, (dd.N, dd.K, P // 2, Q // 2), "y_pooled"), wptr, wbytes,
                                      _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_fwd_relu_pool2")


def conv2d_fwd_1x1_group(d, x, ws_list, bias_list, ys, ws=None, stream=None) -> None:
    """d describes the stacked layer (K = sum of the groups' filter counts); ws_list,
    bias_list (entries or the whole list may be None) and ys are per-group tensors."""
    dd = _desc(d)
    n = len(ws_list)
    if len(ys) != n or (bias_list is not None and len(bias_list) != n):
        raise ValueError("group lists differ in length")
    Ks = [int(w.shape[0]) for w in ws_list]
    karr = (C.c_int32 * n)(*Ks)
    warr = (C.c_void_p * n)(*[_ptr(w, (k, dd.C, 1, 1), "w[%d]" % i) for i, (w, k) in enumerate(zip(ws_list, Ks))])
    yarr = (C.c_void_p * n)(*[_ptr(y, (dd.N, k, dd.H, dd.W), "y[%d]" % i) for i, (y, k) in enumerate(zip(ys, Ks))])
    barr = None
    if bias_list is not None:
        barr = (C.c_void_p * n)(*[_ptr(b, (k,), "bias[%d]" % i) or None for i, (b, k) in enumerate(zip(bias_list, Ks))])
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_FWD, ALGO_IGEMM), stream)
    rc = load().conv2d_fwd_1x1_group(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"), n, karr, warr,
                                     barr, yarr, wptr, wbytes, _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_fwd_1x1_group")


def conv2d_bwd_data(d, dy, w, dx, ws=None, algo: int = ALGO_AUTO, stream=None) -> None:
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_BWD_DATA, algo), stream)
    rc = load().conv2d_bwd_data(C.byref(dd), _ptr(dy, (dd.N, dd.K, P, Q), "dy"),
                                _ptr(w, (dd.K, dd.C, dd.R, dd.S), "w"),
                                _ptr(dx, (dd.N, dd.C, dd.H, dd.W), "dx"), wptr, wbytes, int(algo),
                                _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_bwd_data")


def conv2d_bwd_weight(d, x, dy, dw, dbias=None, scale: float = 1.0, accumulate: bool = False,
                      ws=None, algo: int = ALGO_AUTO, stream=None) -> None:
    dd = _desc(d)
    P, Q = conv2d_output_dims(dd)
    wsb, wptr, wbytes = _ws(ws, conv2d_workspace_bytes(dd, OP_BWD_WEIGHT, algo), stream)
    rc = load().conv2d_bwd_weight(C.byref(dd), _ptr(x, (dd.N, dd.C, dd.H, dd.W), "x"),
                                  _ptr(dy, (dd.N, dd.K, P, Q), "dy"),
                                  _ptr(dw, (dd.K, dd.C, dd.R, dd.S), "dw"),
                                  _ptr(dbias, (dd.K,), "dbias"), float(scale),
                                  1 if accumulate else 0, wptr, wbytes, int(algo), _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_bwd_weight")


def apply_mul_add(x, y, a: float, b: float, stream=None) -> None:
    """y = fl(fl(a*x) + b) per element; x, y device float32 tensors of equal size."""
    n = x.numel()
    if y.numel() != n:
        raise ValueError("x and y differ in size")
    rc = load().apply_mul_add(_ptr(x, None, "x"), _ptr(y, None, "y"), n, float(a), float(b), _stream(stream))
    if rc:
        raise Conv2dError(rc, "apply_mul_add")


# ---- measurement helpers ---------------------------------------------------
def conv2d_profile_begin(capacity: int) -> None:
    rc = load().conv2d_profile_begin(int(capacity))
    if rc:
        raise Conv2dError(rc, "conv2d_profile_begin")


def conv2d_profile_end() -> int:
    return int(load().conv2d_profile_end())


def conv2d_profile_record(i: int):
    """(kernel id, flops, bytes, ms) of recorded launch i; the streams must be synchronised."""
    k, fl, by, ms = C.c_int32(), C.c_double(), C.c_double(), C.c_float()
    rc = load().conv2d_profile_record(int(i), C.byref(k), C.byref(fl), C.byref(by), C.byref(ms))
    if rc:
        raise Conv2dError(rc, "conv2d_profile_record")
    return k.value, fl.value, by.value, ms.value


def conv2d_profile_kernel_name(kernel: int) -> str:
    return load().conv2d_profile_kernel_name(int(kernel)).decode()


def conv2d_probe_mfma_f32(sink, iters: int, stream=None) -> float:
    """Enqueues the pure-MFMA probe; returns the flops it executes."""
    fl = C.c_double()
    rc = load().conv2d_probe_mfma_f32(_ptr(sink, None, "sink"), int(iters), C.byref(fl), _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_probe_mfma_f32")
    return fl.value


def conv2d_probe_copy(src, dst, stream=None) -> None:
    """16-byte-vector copy of src to dst (equal sizes), or a fill of dst when src is None."""
    rc = load().conv2d_probe_copy(_ptr(src, None, "src"), _ptr(dst, None, "dst"), dst.numel(), _stream(stream))
    if rc:
        raise Conv2dError(rc, "conv2d_probe_copy")
