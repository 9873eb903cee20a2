"""ctypes binding of libcvx.so: the same names as include/cvx.h, argument marshalling only.

Every step of the convolution runs in the library's HIP kernels; torch is used here only to hold
device memory and to name the current stream.  There is no CPU or eager fallback: if the shared
library is missing or a GPU call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcvx.so")

CVX_OK = 0
CVX_ERR_NULL, CVX_ERR_BAD_PARAM, CVX_ERR_SHAPE_MISMATCH, CVX_ERR_UNSUPPORTED, CVX_ERR_ALIGNMENT, CVX_ERR_LAUNCH = 1, 2, 3, 4, 5, 6
CVX_F32, CVX_F16, CVX_BF16 = 0, 1, 2
CVX_ACT_IDENTITY, CVX_ACT_RELU, CVX_ACT_LEAKY_RELU, CVX_ACT_TANH, CVX_ACT_LOGISTIC = 0, 1, 2, 3, 4

# Every symbol include/cvx.h declares (checked by the CPU test-suite against the header text).
EXPORTS = [
    "cvx_create", "cvx_set_stream", "cvx_get_stream", "cvx_destroy",
    "cvx_tensor_desc_create", "cvx_tensor_desc_set_4d", "cvx_tensor_desc_get_4d", "cvx_tensor_desc_destroy",
    "cvx_conv_desc_create", "cvx_conv_desc_set_2d", "cvx_conv_desc_set_group_count", "cvx_conv_desc_get_2d",
    "cvx_conv_desc_destroy", "cvx_conv_fwd_output_dim",
    "cvx_conv_fwd", "cvx_conv_fwd_fused", "cvx_conv_fwd_fused_bn",
    "cvx_bias_add", "cvx_activation_fwd", "cvx_conv_fwd_query", "cvx_get_last_kernel", "cvx_set_kernel_policy",
    "cvx_debug_pin_kernel",
    "cvx_status_string", "cvx_last_error",
]


class CvxError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__("%s failed: %s (%d): %s" % (where, _status_name(status), status, detail))
        self.status = status


_lib = None


def lib():
    """The loaded shared library.  Builds it first only when no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, cf, cd = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_double
        pvp, pci = ctypes.POINTER(vp), ctypes.POINTER(ci)
        sig = {
            "cvx_create": [pvp, vp], "cvx_set_stream": [vp, vp], "cvx_get_stream": [vp, pvp], "cvx_destroy": [vp],
            "cvx_tensor_desc_create": [pvp], "cvx_tensor_desc_set_4d": [vp, ci, ci, ci, ci, ci],
            "cvx_tensor_desc_get_4d": [vp, pci, pci, pci, pci, pci], "cvx_tensor_desc_destroy": [vp],
            "cvx_conv_desc_create": [pvp], "cvx_conv_desc_set_2d": [vp, ci, ci, ci, ci, ci, ci],
            "cvx_conv_desc_set_group_count": [vp, ci],
            "cvx_conv_desc_get_2d": [vp, pci, pci, pci, pci, pci, pci, pci], "cvx_conv_desc_destroy": [vp],
            "cvx_conv_fwd_output_dim": [vp, vp, vp, pci, pci, pci, pci],
            "cvx_conv_fwd": [vp, vp, vp, vp, vp, vp, vp, vp],
            "cvx_conv_fwd_fused": [vp, vp, vp, vp, vp, vp, vp, vp, ci, cf, vp, vp],
            "cvx_conv_fwd_fused_bn": [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, cd, ci, cf, vp, vp],
            "cvx_bias_add": [vp, vp, vp, vp, vp], "cvx_activation_fwd": [vp, ci, cf, vp, vp],
            "cvx_conv_fwd_query": [vp, vp, vp, vp, ctypes.c_char_p, ci, ctypes.POINTER(ctypes.c_ulonglong)],
            "cvx_set_kernel_policy": [vp, ci],
            "cvx_get_last_kernel": [vp, ctypes.c_char_p, ci],
            "cvx_debug_pin_kernel": [vp, ctypes.c_char_p],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.argtypes = args
            f.restype = ci
        L.cvx_status_string.argtypes = [ci]
        L.cvx_status_string.restype = ctypes.c_char_p
        L.cvx_last_error.argtypes = []
        L.cvx_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _status_name(st: int) -> str:
    return lib().cvx_status_string(st).decode()


def cvx_status_string(st: int) -> str:
    return _status_name(st)


def cvx_last_error() -> str:
    return lib().cvx_last_error().decode()


def _check(st: int, where: str):
    if st != CVX_OK:
        raise CvxError(st, where, cvx_last_error())


# ---- thin wrappers, one per C function ---------------------------------------------------------
def cvx_create(hip_stream: int = 0) -> int:
    h = ctypes.c_void_p()
    _check(lib().cvx_create(ctypes.byref(h), hip_stream or None), "cvx_create")
    return h.value


def cvx_set_stream(h: int, hip_stream: int) -> None:
    _check(lib().cvx_set_stream(h, hip_stream or None), "cvx_set_stream")


def cvx_get_stream(h: int) -> int:
    s = ctypes.c_void_p()
    _check(lib().cvx_get_stream(h, ctypes.byref(s)), "cvx_get_stream")
    return s.value or 0


def cvx_destroy(h: int) -> None:
    _check(lib().cvx_destroy(h), "cvx_destroy")


def cvx_set_kernel_policy(h: int, policy: int) -> None:
    _check(lib().cvx_set_kernel_policy(h, policy), "cvx_set_kernel_policy")


def cvx_get_last_kernel(h: int) -> str:
    buf = ctypes.create_string_buffer(128)
    _check(lib().cvx_get_last_kernel(h, buf, 128), "cvx_get_last_kernel")
    return buf.value.decode()


def cvx_debug_pin_kernel(h: int, spec: Optional[str]) -> None:
    _check(lib().cvx_debug_pin_kernel(h, spec.encode() if spec else None), "cvx_debug_pin_kernel")


def cvx_tensor_desc_create() -> int:
    t = ctypes.c_void_p()
    _check(lib().cvx_tensor_desc_create(ctypes.byref(t)), "cvx_tensor_desc_create")
    return t.value


def cvx_tensor_desc_set_4d(t: int, dtype: int, n: int, c: int, h: int, w: int) -> None:
    _check(lib().cvx_tensor_desc_set_4d(t, dtype, n, c, h, w), "cvx_tensor_desc_set_4d")


def cvx_tensor_desc_get_4d(t: int) -> Tuple[int, int, int, int, int]:
    v = [ctypes.c_int() for _ in range(5)]
    _check(lib().cvx_tensor_desc_get_4d(t, *[ctypes.byref(x) for x in v]), "cvx_tensor_desc_get_4d")
    return tuple(x.value for x in v)


def cvx_tensor_desc_destroy(t: int) -> None:
    _check(lib().cvx_tensor_desc_destroy(t), "cvx_tensor_desc_destroy")


def cvx_conv_desc_create() -> int:
    c = ctypes.c_void_p()
    _check(lib().cvx_conv_desc_create(ctypes.byref(c)), "cvx_conv_desc_create")
    return c.value


def cvx_conv_desc_set_2d(c: int, pad_h: int, pad_w: int, stride_h: int, stride_w: int, dil_h: int, dil_w: int) -> None:
    _check(lib().cvx_conv_desc_set_2d(c, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w), "cvx_conv_desc_set_2d")


def cvx_conv_desc_set_group_count(c: int, groups: int) -> None:
    _check(lib().cvx_conv_desc_set_group_count(c, groups), "cvx_conv_desc_set_group_count")


def cvx_conv_desc_get_2d(c: int):
    v = [ctypes.c_int() for _ in range(7)]
    _check(lib().cvx_conv_desc_get_2d(c, *[ctypes.byref(x) for x in v]), "cvx_conv_desc_get_2d")
    return tuple(x.value for x in v)


def cvx_conv_desc_destroy(c: int) -> None:
    _check(lib().cvx_conv_desc_destroy(c), "cvx_conv_desc_destroy")


def cvx_conv_fwd_output_dim(c: int, xd: int, wd: int) -> Tuple[int, int, int, int]:
    v = [ctypes.c_int() for _ in range(4)]
    _check(lib().cvx_conv_fwd_output_dim(c, xd, wd, *[ctypes.byref(x) for x in v]), "cvx_conv_fwd_output_dim")
    return tuple(x.value for x in v)


def cvx_conv_fwd(h, xd, x_ptr, wd, w_ptr, conv, yd, y_ptr) -> None:
    _check(lib().cvx_conv_fwd(h, xd, x_ptr, wd, w_ptr, conv, yd, y_ptr), "cvx_conv_fwd")


def cvx_conv_fwd_fused(h, xd, x_ptr, wd, w_ptr, conv, bd, bias_ptr, act, act_alpha, yd, y_ptr) -> None:
    _check(lib().cvx_conv_fwd_fused(h, xd, x_ptr, wd, w_ptr, conv, bd, bias_ptr, act, act_alpha, yd, y_ptr),
           "cvx_conv_fwd_fused")


def cvx_conv_fwd_fused_bn(h, xd, x_ptr, wd, w_ptr, conv, bd, bias_ptr, scale_ptr, shift_ptr, mean_ptr, var_ptr,
                          eps, act, act_alpha, yd, y_ptr) -> None:
    _check(lib().cvx_conv_fwd_fused_bn(h, xd, x_ptr, wd, w_ptr, conv, bd, bias_ptr, scale_ptr, shift_ptr,
                                       mean_ptr, var_ptr, eps, act, act_alpha, yd, y_ptr), "cvx_conv_fwd_fused_bn")


def cvx_bias_add(h, bd, bias_ptr, yd, y_ptr) -> None:
    _check(lib().cvx_bias_add(h, bd, bias_ptr, yd, y_ptr), "cvx_bias_add")


def cvx_activation_fwd(h, act, act_alpha, yd, y_ptr) -> None:
    _check(lib().cvx_activation_fwd(h, act, act_alpha, yd, y_ptr), "cvx_activation_fwd")


def cvx_conv_fwd_query(xd, wd, conv, yd) -> Tuple[str, int]:
    buf = ctypes.create_string_buffer(128)
    ws = ctypes.c_ulonglong()
    _check(lib().cvx_conv_fwd_query(xd, wd, conv, yd, buf, 128, ctypes.byref(ws)), "cvx_conv_fwd_query")
    return buf.value.decode(), ws.value


# ---- torch-tensor convenience layer (still marshalling only) -----------------------------------
def _torch_dtype_code(t) -> int:
    import torch
    return {torch.float32: CVX_F32, torch.float16: CVX_F16, torch.bfloat16: CVX_BF16}[t.dtype]


def _pair(v) -> Tuple[int, int]:
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


class ConvPlan:
    """Descriptors for one convolution problem, created once and reused for every call
    (the create-once / execute-many split of the fusion plan in Sec. V of the MIOpen paper)."""

    def __init__(self, dtype: int, x_shape, w_shape, pad=0, stride=1, dil=1, groups=1,
                 bias_dtype: Optional[int] = None, stream: int = 0, bias_channels: Optional[int] = None):
        self.h = cvx_create(stream)
        self.xd, self.wd, self.yd, self.bd = (cvx_tensor_desc_create() for _ in range(4))
        self.cd = cvx_conv_desc_create()
        cvx_tensor_desc_set_4d(self.xd, dtype, *x_shape)
        cvx_tensor_desc_set_4d(self.wd, dtype, *w_shape)
        cvx_conv_desc_set_2d(self.cd, *_pair(pad), *_pair(stride), *_pair(dil))
        cvx_conv_desc_set_group_count(self.cd, groups)
        self.y_shape = cvx_conv_fwd_output_dim(self.cd, self.xd, self.wd)
        cvx_tensor_desc_set_4d(self.yd, dtype, *self.y_shape)
        cvx_tensor_desc_set_4d(self.bd, dtype if bias_dtype is None else bias_dtype, 1,
                               w_shape[0] if bias_channels is None else bias_channels, 1, 1)
        self.dtype = dtype

    def kernel_name(self) -> str:
        """The kernel the library runs for 16-byte-aligned buffers."""
        return cvx_conv_fwd_query(self.xd, self.wd, self.cd, self.yd)[0]

    def last_kernel(self) -> str:
        return cvx_get_last_kernel(self.h)

    def pin(self, spec: Optional[str]) -> None:
        cvx_debug_pin_kernel(self.h, spec)

    def set_stream(self, stream: int) -> None:
        cvx_set_stream(self.h, stream)

    def run(self, x_ptr: int, w_ptr: int, bias_ptr: Optional[int], y_ptr: int, act: int = CVX_ACT_RELU,
            alpha: float = 0.0) -> None:
        cvx_conv_fwd_fused(self.h, self.xd, x_ptr, self.wd, w_ptr, self.cd, self.bd, bias_ptr, act, alpha,
                           self.yd, y_ptr)

    def run_plain(self, x_ptr: int, w_ptr: int, y_ptr: int) -> None:
        cvx_conv_fwd(self.h, self.xd, x_ptr, self.wd, w_ptr, self.cd, self.yd, y_ptr)

    def run_bn(self, x_ptr, w_ptr, bias_ptr, scale_ptr, shift_ptr, mean_ptr, var_ptr, eps, y_ptr,
               act: int = CVX_ACT_RELU, alpha: float = 0.0) -> None:
        cvx_conv_fwd_fused_bn(self.h, self.xd, x_ptr, self.wd, w_ptr, self.cd, self.bd, bias_ptr, scale_ptr,
                              shift_ptr, mean_ptr, var_ptr, eps, act, alpha, self.yd, y_ptr)

    def close(self) -> None:
        if self.h:
            for d in (self.xd, self.wd, self.yd, self.bd):
                cvx_tensor_desc_destroy(d)
            cvx_conv_desc_destroy(self.cd)
            cvx_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def conv_fwd_fused(x, w, bias=None, *, pad=0, stride=1, dil=1, groups=1, act=CVX_ACT_RELU, alpha=0.0,
                   bn=None, eps=1e-5, out=None, policy: int = 0, pin: Optional[str] = None,
                   info: Optional[dict] = None):
    """y = act(bn(conv(x, w) + bias)) on device tensors (torch, contiguous NCHW).  bn, if given, is a
    tuple (scale, shift, mean, var) of fp32 device tensors with K values each.  Allocates y with
    torch unless `out` is given; everything else happens inside libcvx.so.  `pin` is the developer kernel pin; `info`, if a dict, receives
    the name of the kernel that ran under "kernel"."""
    import torch
    if not (x.is_cuda and w.is_cuda):
        raise ValueError("tensors must live on the GPU; this library has no CPU path")
    if not (x.is_contiguous() and w.is_contiguous()):
        raise ValueError("tensors must be contiguous (packed NCHW / KCRS)")
    dt = _torch_dtype_code(x)
    stream = torch.cuda.current_stream(x.device).cuda_stream
    bias_dt = None if bias is None else _torch_dtype_code(bias)
    if bias is not None and not (bias.is_cuda and bias.is_contiguous()):
        raise ValueError("bias must be a contiguous GPU tensor")
    bias_ch = None if bias is None else bias.numel()
    with ConvPlan(dt, tuple(x.shape), tuple(w.shape), pad, stride, dil, groups, bias_dt, stream, bias_ch) as plan:
        cvx_set_kernel_policy(plan.h, policy)
        if pin:
            plan.pin(pin)
        y = out if out is not None else torch.empty(plan.y_shape, dtype=x.dtype, device=x.device)
        if tuple(y.shape) != tuple(plan.y_shape) or not y.is_contiguous() or y.dtype != x.dtype:
            raise ValueError("out has the wrong shape, dtype or layout")
        bp = None if bias is None else bias.data_ptr()
        if bn is None:
            plan.run(x.data_ptr(), w.data_ptr(), bp, y.data_ptr(), act, alpha)
        else:
            sc, sh, mu, var = bn
            plan.run_bn(x.data_ptr(), w.data_ptr(), bp, sc.data_ptr(), sh.data_ptr(), mu.data_ptr(), var.data_ptr(),
                        eps, y.data_ptr(), act, alpha)
        if info is not None:
            info["kernel"] = plan.last_kernel()
    return y
