"""Thin ctypes binding of the shflbw C ABI (see ``include/shflbw.h``).

Argument marshalling only: every step of the hot path runs inside the
library's kernels.  torch tensors are used for device memory and for the
stream handle; numpy arrays for host-side inputs of the compressor.

The library is required: if ``libshflbw.so`` has not been built this module
raises at first use.  There is no CPU fallback.
"""
import ctypes
import os

import numpy as np

F16, BF16, F32 = 0, 1, 2
NCHW, CHWN = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshflbw.so")
_lib = None

EXPORTS = [
    "shflbw_compress", "shflbw_pattern_search", "shflbw_destroy", "shflbw_info", "shflbw_row_indices",
    "shflbw_group_columns", "shflbw_decompress", "shflbw_device_bytes", "shflbw_bind_device",
    "shflbw_set_tuning", "shflbw_device_status", "shflbw_set_wait_limit", "shflbw_spmm", "shflbw_spmm_unbound",
    "shflbw_conv2d",
    "shflbw_layernorm_transpose", "shflbw_status_string", "shflbw_last_error", "shflbw_last_kernel",
]


class ShflbwError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("shflbw status %d (%s): %s" % (status, status_string(status), text))
        self.status = status


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2203_05016_amd.build`"
                               % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.shflbw_compress.restype = i32
        L.shflbw_compress.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, ctypes.POINTER(vp)]
        L.shflbw_destroy.restype = None
        L.shflbw_destroy.argtypes = [vp]
        L.shflbw_info.restype = i32
        L.shflbw_info.argtypes = [vp] + [ctypes.POINTER(i32)] * 4 + \
            [ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
        L.shflbw_row_indices.restype = i32
        L.shflbw_row_indices.argtypes = [vp, vp]
        L.shflbw_group_columns.restype = i32
        L.shflbw_group_columns.argtypes = [vp, i32, vp, i32]
        L.shflbw_decompress.restype = i32
        L.shflbw_decompress.argtypes = [vp, vp, i32]
        L.shflbw_device_bytes.restype = ctypes.c_size_t
        L.shflbw_device_bytes.argtypes = [vp]
        L.shflbw_bind_device.restype = i32
        L.shflbw_bind_device.argtypes = [vp, vp, vp]
        L.shflbw_set_tuning.restype = i32
        L.shflbw_set_tuning.argtypes = [vp, i32, i32]
        L.shflbw_device_status.restype = i32
        L.shflbw_device_status.argtypes = [vp, vp]
        L.shflbw_set_wait_limit.restype = i32
        L.shflbw_set_wait_limit.argtypes = [vp, i32]
        L.shflbw_spmm.restype = i32
        L.shflbw_spmm.argtypes = [vp, vp, i64, vp, i64, i64, i32, vp]
        L.shflbw_spmm_unbound.restype = i32
        L.shflbw_spmm_unbound.argtypes = [vp, vp, i64, vp, i64, i64, i32, vp]
        L.shflbw_conv2d.restype = i32
        L.shflbw_conv2d.argtypes = [vp, vp, vp] + [i32] * 10 + [i32, i32, vp]
        L.shflbw_pattern_search.restype = i32
        L.shflbw_pattern_search.argtypes = [vp, i32, i32, i32, i32, ctypes.c_double, ctypes.c_double,
                                            i32, i32, vp, vp]
        L.shflbw_layernorm_transpose.restype = i32
        L.shflbw_layernorm_transpose.argtypes = [vp, i64, vp, vp, ctypes.c_float, i32, vp, i64, i64,
                                                 i32, i32, vp]
        L.shflbw_status_string.restype = ctypes.c_char_p
        L.shflbw_status_string.argtypes = [i32]
        L.shflbw_last_error.restype = ctypes.c_char_p
        L.shflbw_last_error.argtypes = []
        L.shflbw_last_kernel.restype = ctypes.c_char_p
        L.shflbw_last_kernel.argtypes = []
        _lib = L
    return _lib


def status_string(status):
    return lib().shflbw_status_string(int(status)).decode()


def last_error():
    return lib().shflbw_last_error().decode()


def last_kernel():
    """Name of the kernel this thread's last spmm / conv2d call launched."""
    return lib().shflbw_last_kernel().decode()


def _check(rc):
    if rc < 0:
        raise ShflbwError(rc, last_error())
    return rc


def _host_ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


_YDTYPE = None   # torch dtype -> shflbw_dtype, filled on first use (torch is imported lazily)


def _ydtype(t):
    global _YDTYPE
    if _YDTYPE is None:
        import torch
        _YDTYPE = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}
    try:
        return _YDTYPE[t.dtype]
    except KeyError:
        raise TypeError("output tensor must be float16, bfloat16 or float32") from None


class Matrix:
    """Owner of one ``shflbw_matrix`` handle and, once bound, of the device
    buffer (a torch uint8 tensor) that holds its packed arrays."""

    def __init__(self, handle, bf16=False):
        self._h = handle
        self._dev = None
        self.bf16 = bf16   # operand format: bfloat16 instead of float16
        self._info = None  # what shflbw_info reports: fixed once the matrix is packed
        self._odt = None

    def _operand_dtype(self):
        if self._odt is None:
            import torch
            self._odt = torch.bfloat16 if self.bf16 else torch.float16
        return self._odt

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.shflbw_destroy(h)

    # -- host side
    def info(self):
        if self._info is None:
            M, K, V, G = (ctypes.c_int() for _ in range(4))
            nnz, sp = ctypes.c_int64(), ctypes.c_double()
            _check(lib().shflbw_info(self._h, M, K, V, G, nnz, sp))
            self._info = dict(M=M.value, K=K.value, V=V.value, groups=G.value, nnz=nnz.value,
                              sparsity=sp.value)
        return dict(self._info)

    def row_indices(self):
        out = np.empty(self.info()["M"], dtype=np.int32)
        _check(lib().shflbw_row_indices(self._h, _host_ptr(out)))
        return out

    def group_columns(self, g):
        n = _check(lib().shflbw_group_columns(self._h, g, None, 0))
        out = np.empty(n, dtype=np.int32)
        if n:
            _check(lib().shflbw_group_columns(self._h, g, _host_ptr(out), n))
        return out

    def decompress(self, ldw=None):
        i = self.info()
        ldw = i["K"] if ldw is None else ldw
        out = np.zeros((i["M"], ldw), dtype=np.uint16 if self.bf16 else np.float16)
        _check(lib().shflbw_decompress(self._h, _host_ptr(out), ldw))
        return out

    def device_bytes(self):
        return int(lib().shflbw_device_bytes(self._h))

    def set_tuning(self, kernel=0, tile_n=0):
        _check(lib().shflbw_set_tuning(self._h, kernel, tile_n))

    def set_wait_limit(self, tries):
        _check(lib().shflbw_set_wait_limit(self._h, tries))

    def device_status(self, stream=None):
        """Waits for the stream; raises ShflbwError (status -10) if a bounded wait of
        the slab kernel ran out in a launch on this matrix since the last call."""
        _check(lib().shflbw_device_status(self._h, _stream_ptr(stream)))

    # -- device side
    def bind_device(self, device="cuda:0", stream=None):
        import torch
        buf = torch.empty(self.device_bytes(), dtype=torch.uint8, device=device)
        _check(lib().shflbw_bind_device(self._h, ctypes.c_void_p(buf.data_ptr()),
                                        _stream_ptr(stream)))
        self._dev = buf
        return self

    def _require_on_bound_device(self, t, what):
        """The C ABI takes bare addresses: it cannot tell a host tensor, or one on
        another GPU, from device memory of the GPU the matrix is bound to."""
        if self._dev is None:
            raise RuntimeError("call bind_device before %s" % what)
        if not t.is_cuda or t.device != self._dev.device:
            raise ValueError("%s must live on %s, where the matrix is bound (got %s)"
                             % (what, self._dev.device, t.device))

    def spmm(self, X, Y=None, out_dtype=None, stream=None):
        """Y = (W . mask) X for a device tensor X of shape (K, N) in the
        matrix's operand format (float16, or bfloat16).  The C ABI has no K
        argument and sees only addresses, so shapes, strides and devices are
        checked here, before anything is enqueued."""
        if X.dtype != self._operand_dtype() or X.dim() != 2 or X.stride(1) != 1 and X.shape[1] > 1:
            raise TypeError("X must be a 2-D %s tensor with unit column stride" % self._operand_dtype())
        info = self.info()
        K, N = X.shape
        if K != info["K"]:
            raise ValueError("X has %d rows, the packed matrix has K = %d columns" % (K, info["K"]))
        if K > 1 and X.stride(0) < N:
            raise ValueError("rows of X overlap (row stride %d < N = %d)" % (X.stride(0), N))
        if Y is not None:
            if Y.dim() != 2 or tuple(Y.shape) != (info["M"], N):
                raise ValueError("Y must have shape (%d, %d), got %r" % (info["M"], N, tuple(Y.shape)))
            if N > 1 and Y.stride(1) != 1:
                raise ValueError("Y must have unit column stride")
            if Y.shape[0] > 1 and Y.stride(0) < N:
                raise ValueError("rows of Y overlap (row stride %d < N = %d)" % (Y.stride(0), N))
            _ydtype(Y)
        self._require_on_bound_device(X, "X")
        if Y is None:
            import torch
            Y = torch.empty((info["M"], N), dtype=out_dtype or self._operand_dtype(),
                            device=X.device)
        else:
            self._require_on_bound_device(Y, "Y")
        ldx = X.stride(0) if K > 1 else max(N, 1)
        ldy = Y.stride(0) if Y.shape[0] > 1 else max(N, 1)
        rc = lib().shflbw_spmm(self._h, X.data_ptr(), ldx, Y.data_ptr(), ldy, N, _ydtype(Y),
                               _stream_ptr(stream))
        if rc < 0:
            _check(rc)
        return Y

    def conv2d(self, inp, R, S, stride=(1, 1), pad=(0, 0), layout="NCHW", out=None,
               out_dtype=None, stream=None):
        """Masked conv2d of a contiguous device tensor in the matrix's operand format."""
        import torch
        if inp.dtype != self._operand_dtype() or not inp.is_contiguous() or inp.dim() != 4:
            raise TypeError("input must be a contiguous 4-D %s tensor" % self._operand_dtype())
        if layout not in ("NCHW", "CHWN"):
            raise ValueError("layout must be 'NCHW' or 'CHWN'")
        if layout == "NCHW":
            B, C, H, W = inp.shape
        else:
            C, H, W, B = inp.shape
        info = self.info()
        if C * R * S != info["K"]:
            raise ValueError("C_in*R*S = %d does not match the packed matrix's K = %d" % (C * R * S, info["K"]))
        if min(stride) < 1 or min(pad) < 0 or H + 2 * pad[0] < R or W + 2 * pad[1] < S:
            raise ValueError("bad stride, padding or kernel size")
        Ho = (H + 2 * pad[0] - R) // stride[0] + 1
        Wo = (W + 2 * pad[1] - S) // stride[1] + 1
        Cout = info["M"]
        shape = (B, Cout, Ho, Wo) if layout == "NCHW" else (Cout, Ho, Wo, B)
        if out is not None:
            if tuple(out.shape) != shape or not out.is_contiguous():
                raise ValueError("out must be a contiguous tensor of shape %r, got %r" % (shape, tuple(out.shape)))
            _ydtype(out)
        self._require_on_bound_device(inp, "input")
        if out is None:
            out = torch.empty(shape, dtype=out_dtype or self._operand_dtype(), device=inp.device)
        else:
            self._require_on_bound_device(out, "out")
        _check(lib().shflbw_conv2d(self._h, inp.data_ptr(), out.data_ptr(), B, C, H, W, R, S,
                                   stride[0], stride[1], pad[0], pad[1],
                                   NCHW if layout == "NCHW" else CHWN, _ydtype(out),
                                   _stream_ptr(stream)))
        return out


def compress(W, mask, perm, V, K=None):
    """shflbw_compress on numpy arrays: W (M, ldw) float16, or uint16 holding
    bfloat16 bit patterns (numpy has no such dtype), of which the first K
    columns are the matrix (default: all), mask (M, K) uint8 or None, perm
    (M,) int32 or None."""
    if W.dtype not in (np.float16, np.uint16) or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array, or uint16 holding bfloat16 bits")
    bf16 = W.dtype == np.uint16
    W = np.ascontiguousarray(W)
    M, ldw = W.shape
    K = ldw if K is None else K
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    p = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    if m is not None and m.shape != (M, K):
        raise ValueError("mask shape")
    if p is not None and p.shape != (M,):
        raise ValueError("perm shape")
    h = ctypes.c_void_p()
    _check(lib().shflbw_compress(_host_ptr(W), ldw, _host_ptr(m), _host_ptr(p), M, K, V,
                                 BF16 if bf16 else F16, ctypes.byref(h)))
    return Matrix(h, bf16)


def layernorm_transpose(x, gamma=None, beta=None, eps=1e-5, normalize=True, out=None, stream=None):
    """shflbw_layernorm_transpose on device tensors: x (N tokens, K features)
    float16 or bfloat16 with unit feature stride; returns the (K, N) matrix
    shflbw_spmm takes as X."""
    import torch
    if x.dtype not in (torch.float16, torch.bfloat16) or x.dim() != 2 or x.stride(1) != 1:
        raise TypeError("x must be a 2-D float16 or bfloat16 tensor with unit feature stride")
    N, K = x.shape
    for t in (gamma, beta):
        if t is not None and (t.dtype != x.dtype or t.shape != (K,) or not t.is_contiguous()):
            raise TypeError("gamma and beta must be contiguous (K,) tensors of x's dtype")
    if out is None:
        out = torch.empty((K, N), dtype=x.dtype, device=x.device)
    if out.dtype != x.dtype or out.shape != (K, N) or out.stride(1) != 1:
        raise TypeError("out must be a (K, N) tensor of x's dtype with unit token stride")
    for t in (x, out, gamma, beta):
        if t is not None and (not t.is_cuda or t.device != x.device):
            raise ValueError("x, gamma, beta and out must live on one GPU")
    if (N > 1 and x.stride(0) < K) or (K > 1 and out.stride(0) < N):
        raise ValueError("rows of x or out overlap")
    ptr = lambda t: ctypes.c_void_p(None if t is None else t.data_ptr())
    _check(lib().shflbw_layernorm_transpose(ptr(x), x.stride(0) if N > 1 else K, ptr(gamma), ptr(beta),
                                            float(eps), 1 if normalize else 0, ptr(out),
                                            out.stride(0) if K > 1 else N, N, K,
                                            BF16 if x.dtype == torch.bfloat16 else F16,
                                            _stream_ptr(stream)))
    return out


def pattern_search(W, V, alpha, beta=None, iterations=10):
    """shflbw_pattern_search on a numpy matrix (float16, or uint16 holding
    bfloat16 bit patterns): returns (perm, mask) ready for ``compress``.
    beta None = the paper's 2*alpha."""
    if W.dtype not in (np.float16, np.uint16) or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array, or uint16 holding bfloat16 bits")
    W = np.ascontiguousarray(W)
    M, K = W.shape
    perm = np.empty(M, dtype=np.int32)
    mask = np.empty((M, K), dtype=np.uint8)
    _check(lib().shflbw_pattern_search(_host_ptr(W), K, M, K, V, float(alpha),
                                       -1.0 if beta is None else float(beta), int(iterations),
                                       BF16 if W.dtype == np.uint16 else F16,
                                       _host_ptr(perm), _host_ptr(mask)))
    return perm, mask
