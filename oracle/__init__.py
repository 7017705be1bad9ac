"""ctypes front end of the CPU oracle (``sw_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports this package and
this package never imports the GPU library.

Every function takes numpy arrays, widens nothing itself (the C code widens
fp32 to fp64 exactly) and returns ``(y, D)`` in float64, where ``D`` is the
per-output magnitude sum ``sum |x*w|`` that the parity tolerance is relative
to.  The int8 function returns exact int32 sums.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sw_oracle.c")
_LIB = os.path.join(_HERE, "libsw_oracle.so")
_lib = None

POOL_AVG = 0
POOL_MAX = 1


def build(force: bool = False) -> str:
    """Compile ``sw_oracle.c`` with the host gcc (no fast-math) and return the path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    lib.oracle_out_dim.restype = i64
    lib.oracle_out_dim.argtypes = [i64] * 4
    lib.oracle_max_threads.restype = ctypes.c_int
    lib.oracle_set_threads.argtypes = [ctypes.c_int]
    lib.oracle_conv2d.restype = ctypes.c_int
    lib.oracle_conv2d.argtypes = [vp] * 4 + [i64] * 9
    lib.oracle_conv2d_depthwise.restype = ctypes.c_int
    lib.oracle_conv2d_depthwise.argtypes = [vp] * 4 + [i64] * 8
    lib.oracle_conv1d.restype = ctypes.c_int
    lib.oracle_conv1d.argtypes = [vp] * 4 + [i64] * 5
    lib.oracle_pool1d.restype = ctypes.c_int
    lib.oracle_pool1d.argtypes = [vp] * 3 + [i64] * 4 + [ctypes.c_int]
    lib.oracle_pool2d.restype = ctypes.c_int
    lib.oracle_pool2d.argtypes = [vp] * 3 + [i64] * 7 + [ctypes.c_int]
    lib.oracle_requant_s8.restype = ctypes.c_int
    lib.oracle_requant_s8.argtypes = [vp] * 4 + [i64] * 3 + [ctypes.c_int]
    lib.oracle_out_dim_dilated.restype = i64
    lib.oracle_out_dim_dilated.argtypes = [i64] * 5
    lib.oracle_conv2d_dilated.restype = ctypes.c_int
    lib.oracle_conv2d_dilated.argtypes = [vp] * 4 + [i64] * 10 + [ctypes.c_int]
    lib.oracle_bias_relu.restype = ctypes.c_int
    lib.oracle_bias_relu.argtypes = [vp] * 3 + [i64] * 3 + [ctypes.c_int]
    lib.oracle_conv2d_s8.restype = ctypes.c_int
    lib.oracle_conv2d_s8.argtypes = [vp] * 3 + [i64] * 9
    _lib = lib
    return lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _as(a, dtype, ndim) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    if a.ndim != ndim:
        raise ValueError(f"expected {ndim} dimensions, got shape {a.shape}")
    return a


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 values they denote (exact): the widening the 16-bit entry points are
    defined on."""
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_rne(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even; finite inputs."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def f16_to_f32(h: np.ndarray) -> np.ndarray:
    """IEEE half-precision bit patterns (uint16) -> the fp32 values they denote (exact; numpy's own widening)."""
    return np.ascontiguousarray(h, np.uint16).view(np.float16).astype(np.float32)


def out_dim(n_in: int, k: int, stride: int, pad: int) -> int:
    return int(_load().oracle_out_dim(n_in, k, stride, pad))


def conv2d(x, w, stride: int = 1, pad: int = 0):
    x = _as(x, np.float32, 4)
    w = _as(w, np.float32, 4)
    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch")
    Ho, Wo = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("filter does not fit the padded input")
    y = np.empty((N, C_out, Ho, Wo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_conv2d(_p(x), _p(w), _p(y), _p(d), N, C_in, C_out, H, W, R, S, stride, pad)
    if rc:
        raise ValueError(f"oracle_conv2d rejected the arguments (code {rc})")
    return y, d


def conv2d_depthwise(x, w, stride: int = 1, pad: int = 0):
    x = _as(x, np.float32, 4)
    w = _as(w, np.float32, 4)
    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    Ho, Wo = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("filter does not fit the padded input")
    y = np.empty((N, C, Ho, Wo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_conv2d_depthwise(_p(x), _p(w), _p(y), _p(d), N, C, H, W, R, S, stride, pad)
    if rc:
        raise ValueError(f"oracle_conv2d_depthwise rejected the arguments (code {rc})")
    return y, d


def conv1d(x, w, stride: int = 1, pad: int = 0):
    x = _as(x, np.float32, 2)
    w = _as(w, np.float32, 1)
    rows, length = x.shape
    k = w.shape[0]
    Lo = out_dim(length, k, stride, pad)
    if Lo <= 0:
        raise ValueError("filter does not fit the padded input")
    y = np.empty((rows, Lo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_conv1d(_p(x), _p(w), _p(y), _p(d), rows, length, k, stride, pad)
    if rc:
        raise ValueError(f"oracle_conv1d rejected the arguments (code {rc})")
    return y, d


def pool1d(x, window: int, stride: int = 1, mode: int = POOL_AVG):
    x = _as(x, np.float32, 2)
    rows, length = x.shape
    Lo = out_dim(length, window, stride, 0)
    if Lo <= 0:
        raise ValueError("window does not fit the input")
    y = np.empty((rows, Lo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_pool1d(_p(x), _p(y), _p(d), rows, length, window, stride, mode)
    if rc:
        raise ValueError(f"oracle_pool1d rejected the arguments (code {rc})")
    return y, d


def pool2d(x, R: int, S: int, stride: int = 1, pad: int = 0, mode: int = POOL_AVG):
    """x [N, C, H, W] -> (y, D) [N, C, H_out, W_out]; average over zero padding with divisor R*S,
    maximum over the positions inside the plane."""
    x = _as(x, np.float32, 4)
    N, C, H, W = x.shape
    Ho, Wo = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("window does not fit the padded input")
    y = np.empty((N, C, Ho, Wo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_pool2d(_p(x), _p(y), _p(d), N * C, H, W, R, S, stride, pad, mode)
    if rc:
        raise ValueError(f"oracle_pool2d rejected the arguments (code {rc})")
    return y, d


def conv2d_s8(x, w, stride: int = 1, pad: int = 0):
    x = _as(x, np.int8, 4)
    w = _as(w, np.int8, 4)
    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch")
    Ho, Wo = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("filter does not fit the padded input")
    y = np.empty((N, C_out, Ho, Wo), np.int32)
    rc = _load().oracle_conv2d_s8(_p(x), _p(w), _p(y), N, C_in, C_out, H, W, R, S, stride, pad)
    if rc == 2:
        raise OverflowError("an exact sum does not fit int32")
    if rc:
        raise ValueError(f"oracle_conv2d_s8 rejected the arguments (code {rc})")
    return y


def conv2d_s8_requant(x, w, bias, scale, stride: int = 1, pad: int = 0, relu: bool = False):
    """int8 convolution followed by per-channel requantisation to int8:
    q = clamp(rne(scale[co] * float(acc + bias[co])), 0 if relu else -128, 127); bias int32 [C_out] or None."""
    acc = conv2d_s8(x, w, stride, pad)
    N, C_out, Ho, Wo = acc.shape
    scale = _as(scale, np.float32, 1)
    if scale.shape[0] != C_out:
        raise ValueError("one scale per output channel")
    if bias is not None:
        bias = _as(bias, np.int32, 1)
        if bias.shape[0] != C_out:
            raise ValueError("one bias per output channel")
    q = np.empty(acc.shape, np.int8)
    rc = _load().oracle_requant_s8(_p(acc), _p(bias) if bias is not None else None, _p(scale), _p(q),
                                   N, C_out, Ho * Wo, 1 if relu else 0)
    if rc == 2:
        raise OverflowError("sum plus bias does not fit int32")
    if rc:
        raise ValueError(f"oracle_requant_s8 rejected the arguments (code {rc})")
    return q


def conv2d_bias_relu(x, w, bias, stride: int = 1, pad: int = 0, relu: bool = False):
    """fp32 convolution followed by a per-channel bias and an optional rectifier, in fp64:
    y = act(conv2d(x, w) + bias[co]); returns (y, D) with D = sum|x*w| + |bias[co]|.  bias fp32 [C_out] or None."""
    y, d = conv2d(x, w, stride, pad)
    N, C_out, Ho, Wo = y.shape
    if bias is not None:
        bias = _as(bias, np.float32, 1)
        if bias.shape[0] != C_out:
            raise ValueError("one bias per output channel")
    rc = _load().oracle_bias_relu(_p(y), _p(d), _p(bias) if bias is not None else None, N, C_out, Ho * Wo,
                                  1 if relu else 0)
    if rc:
        raise ValueError(f"oracle_bias_relu rejected the arguments (code {rc})")
    return y, d


def conv2d_dilated(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, depthwise: bool = False):
    """Dilated convolution in fp64: taps `dilation` positions apart.  x [N,C_in,H,W]; w [C_out,C_in,R,S], or
    [C,1,R,S] with depthwise=True.  Returns (y, D)."""
    x = _as(x, np.float32, 4)
    w = _as(w, np.float32, 4)
    N, C_in, H, W = x.shape
    C_out, Cw, R, S = w.shape
    if (depthwise and (Cw != 1 or C_out != C_in)) or (not depthwise and Cw != C_in):
        raise ValueError("channel mismatch between x and w")
    if dilation < 1:
        raise ValueError("dilation must be at least 1")
    Ho = int(_load().oracle_out_dim_dilated(H, R, stride, pad, dilation))
    Wo = int(_load().oracle_out_dim_dilated(W, S, stride, pad, dilation))
    if Ho <= 0 or Wo <= 0:
        raise ValueError("the dilated filter does not fit the padded input")
    y = np.empty((N, C_out, Ho, Wo), np.float64)
    d = np.empty_like(y)
    rc = _load().oracle_conv2d_dilated(_p(x), _p(w), _p(y), _p(d), N, C_in, C_out, H, W, R, S, stride, pad,
                                       dilation, 1 if depthwise else 0)
    if rc:
        raise ValueError(f"oracle_conv2d_dilated rejected the arguments (code {rc})")
    return y, d


def conv2d_depthwise_bias_relu(x, w, bias, stride: int = 1, pad: int = 0, relu: bool = False):
    """Depthwise convolution followed by a per-channel bias and an optional rectifier, in fp64 (the same
    oracle_bias_relu step as conv2d_bias_relu).  Returns (y, D) with D = sum|x*w| + |bias[c]|."""
    y, d = conv2d_depthwise(x, w, stride, pad)
    N, C, Ho, Wo = y.shape
    if bias is not None:
        bias = _as(bias, np.float32, 1)
        if bias.shape[0] != C:
            raise ValueError("one bias per channel")
    rc = _load().oracle_bias_relu(_p(y), _p(d), _p(bias) if bias is not None else None, N, C, Ho * Wo,
                                  1 if relu else 0)
    if rc:
        raise ValueError(f"oracle_bias_relu rejected the arguments (code {rc})")
    return y, d


def conv2d_s8_nhwc(x, w, stride: int = 1, pad: int = 0):
    """The int8 convolution on channel-last tensors: x [N,H,W,C_in], w [C_out,R,S,C_in] -> y [N,H_out,W_out,C_out]
    int32.  Only the axes are permuted around conv2d_s8 (a change of layout, no arithmetic)."""
    x = _as(x, np.int8, 4)
    w = _as(w, np.int8, 4)
    y = conv2d_s8(np.ascontiguousarray(x.transpose(0, 3, 1, 2)), np.ascontiguousarray(w.transpose(0, 3, 1, 2)),
                  stride, pad)
    return np.ascontiguousarray(y.transpose(0, 2, 3, 1))


def conv2d_s8_nhwc_requant(x, w, bias, scale, stride: int = 1, pad: int = 0, relu: bool = False):
    """conv2d_s8_requant on channel-last tensors (axes permuted, no arithmetic added)."""
    x = _as(x, np.int8, 4)
    w = _as(w, np.int8, 4)
    q = conv2d_s8_requant(np.ascontiguousarray(x.transpose(0, 3, 1, 2)), np.ascontiguousarray(w.transpose(0, 3, 1, 2)),
                          bias, scale, stride, pad, relu)
    return np.ascontiguousarray(q.transpose(0, 2, 3, 1))


def conv2d_nhwc(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False):
    """The fp32 convolution on channel-last tensors, in fp64: x [N,H,W,C_in], w [C_out,R,S,C_in] ->
    (y, D) [N,H_out,W_out,C_out], y = act(conv + bias[co]).  Only the axes are permuted around conv2d_dilated and
    the oracle_bias_relu step (a change of layout, no arithmetic of its own)."""
    x = _as(x, np.float32, 4)
    w = _as(w, np.float32, 4)
    y, d = conv2d_dilated(np.ascontiguousarray(x.transpose(0, 3, 1, 2)), np.ascontiguousarray(w.transpose(0, 3, 1, 2)),
                          stride, pad, dilation)
    if bias is not None or relu:
        N, C_out, Ho, Wo = y.shape
        if bias is not None:
            bias = _as(bias, np.float32, 1)
            if bias.shape[0] != C_out:
                raise ValueError("one bias per output channel")
        rc = _load().oracle_bias_relu(_p(y), _p(d), _p(bias) if bias is not None else None, N, C_out, Ho * Wo,
                                      1 if relu else 0)
        if rc:
            raise ValueError(f"oracle_bias_relu rejected the arguments (code {rc})")
    return np.ascontiguousarray(y.transpose(0, 2, 3, 1)), np.ascontiguousarray(d.transpose(0, 2, 3, 1))


def conv2d_bf16_nhwc(x_bits, w_bits, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False):
    """The same for bf16 tensors given as bit patterns (uint16): both are widened to fp32 (exact), the sums are
    taken in fp64; returns the unrounded (y, D) -- the one rounding of the finished sum to bf16 is the caller's
    to account for (f32_to_bf16_rne gives the nearest-even pattern)."""
    return conv2d_nhwc(bf16_to_f32(np.asarray(x_bits, np.uint16)), bf16_to_f32(np.asarray(w_bits, np.uint16)), stride, pad,
                       dilation, bias, relu)


def conv2d_f16_nhwc(x_bits, w_bits, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False):
    """The same for IEEE half-precision tensors given as bit patterns (uint16): both are widened to fp32 (exact), the
    sums are taken in fp64; returns the unrounded (y, D) -- the one rounding of the finished sum to half precision
    (nearest even: numpy's astype(float16)) is the caller's to account for."""
    return conv2d_nhwc(f16_to_f32(np.asarray(x_bits, np.uint16)), f16_to_f32(np.asarray(w_bits, np.uint16)), stride, pad,
                       dilation, bias, relu)


def dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, relu_dw: bool = True, relu_pw: bool = False):
    """A depthwise-separable block in fp64: t = act_dw(depthwise3x3(x, stride 1, pad 1) + b_dw), then
    y = act_pw(sum_c w_pw[co, c] * t[c] + b_pw[co]).  The depthwise stage is conv2d_depthwise_bias_relu; the pointwise
    stage is a plain matrix product over the channels (numpy, fp64).  Returns (y, D): D is the magnitude sum of the
    composite, sum_c |w_pw[co, c]| * D_dw[c] + |b_pw[co]|, the scale the parity tolerance is relative to."""
    w_dw = _as(w_dw, np.float32, 4)
    w_pw = _as(w_pw, np.float32, 4)
    if w_dw.shape[1:] != (1, 3, 3) or w_pw.shape[2:] != (1, 1) or w_pw.shape[1] != w_dw.shape[0]:
        raise ValueError("w_dw must be [C,1,3,3] and w_pw [C_out,C,1,1]")
    t, d_t = conv2d_depthwise_bias_relu(x, w_dw, b_dw, 1, 1, relu_dw)
    m = w_pw[:, :, 0, 0].astype(np.float64)
    y = np.einsum("oc,nchw->nohw", m, t)
    d = np.einsum("oc,nchw->nohw", np.abs(m), d_t)
    if b_pw is not None:
        b = _as(b_pw, np.float32, 1).astype(np.float64)
        if b.shape[0] != m.shape[0]:
            raise ValueError("one pointwise bias per output channel")
        y += b[None, :, None, None]
        d += np.abs(b)[None, :, None, None]
    if relu_pw:
        y = np.maximum(y, 0.0)
    return y, d
