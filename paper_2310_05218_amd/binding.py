"""Thin ctypes binding of libswconv.so: argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the computation runs in
the library's kernels.  The functions carry the names of the C entry points they call.  If the
library has not been built they raise: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libswconv.so")

SW_OK = 0
SW_ERR_NULL, SW_ERR_SHAPE, SW_ERR_UNSUPPORTED, SW_ERR_ALIGN, SW_ERR_ALIAS, SW_ERR_LAUNCH, SW_ERR_JIT = 1, 2, 3, 4, 5, 6, 7
SW_POOL_AVG, SW_POOL_MAX = 0, 1

EXPORTS = ("sw_conv1d", "sw_pool1d", "sw_pool2d", "sw_conv2d", "sw_conv2d_depthwise", "sw_conv2d_s8",
           "sw_conv2d_s8_requant", "sw_conv2d_s8_nhwc", "sw_conv2d_s8_nhwc_requant", "sw_conv2d_nhwc", "sw_conv2d_bf16_nhwc", "sw_conv2d_f16_nhwc", "sw_conv2d_bias_relu", "sw_dw_pw_block", "sw_conv2d_depthwise_bias_relu", "sw_conv2d_dilated", "sw_conv2d_depthwise_dilated",
           "sw_conv2d_depthwise_bf16", "sw_conv2d_depthwise_jit", "sw_jit_prepare_depthwise", "sw_jit_compile_check",
           "sw_conv2d_depthwise_dilated_jit", "sw_jit_prepare_depthwise_dilated", "sw_jit_compile_check_dilated",
           "sw_jit_cached_kernels",
           "sw_s8_packed_filter_bytes", "sw_s8_pack_filter", "sw_conv2d_s8_packed", "sw_conv2d_s8_packed_requant",
           "sw_probe", "sw_probe_ops", "sw_out_dim", "sw_out_dim_dilated", "sw_workspace_bytes", "sw_status_string", "sw_version", "sw_last_kernel")

_lib = None


class SwError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libswconv.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2310_05218_amd.build` first")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.sw_conv1d.restype = i32
    L.sw_conv1d.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp]
    L.sw_pool1d.restype = i32
    L.sw_pool1d.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp]
    L.sw_pool2d.restype = i32
    L.sw_pool2d.argtypes = [vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d.restype = i32
    L.sw_conv2d.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d_bias_relu.restype = i32
    L.sw_conv2d_bias_relu.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp]
    L.sw_conv2d_depthwise_bias_relu.restype = i32
    L.sw_conv2d_depthwise_bias_relu.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_dw_pw_block.restype = i32
    L.sw_dw_pw_block.argtypes = [vp] * 6 + [i32] * 7 + [vp]
    L.sw_conv2d_dilated.restype = i32
    L.sw_conv2d_dilated.argtypes = [vp, vp, vp] + [i32] * 10 + [vp]
    L.sw_conv2d_depthwise_dilated.restype = i32
    L.sw_conv2d_depthwise_dilated.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d_depthwise.restype = i32
    L.sw_conv2d_depthwise.argtypes = [vp, vp, vp] + [i32] * 8 + [vp]
    L.sw_conv2d_depthwise_bf16.restype = i32
    L.sw_conv2d_depthwise_bf16.argtypes = [vp, vp, vp] + [i32] * 8 + [vp]
    L.sw_conv2d_depthwise_jit.restype = i32
    L.sw_conv2d_depthwise_jit.argtypes = [vp, vp, vp] + [i32] * 8 + [vp]
    for name in ("sw_jit_prepare_depthwise", "sw_jit_compile_check"):
        getattr(L, name).restype = i32
        getattr(L, name).argtypes = [i32] * 6
    L.sw_conv2d_depthwise_dilated_jit.restype = i32
    L.sw_conv2d_depthwise_dilated_jit.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    for name in ("sw_jit_prepare_depthwise_dilated", "sw_jit_compile_check_dilated"):
        getattr(L, name).restype = i32
        getattr(L, name).argtypes = [i32] * 7
    L.sw_jit_cached_kernels.restype = i32
    L.sw_jit_cached_kernels.argtypes = []
    L.sw_conv2d_s8.restype = i32
    L.sw_conv2d_s8.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d_s8_nhwc.restype = i32
    L.sw_conv2d_s8_nhwc.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d_nhwc.restype = i32
    L.sw_conv2d_nhwc.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [vp]
    L.sw_conv2d_bf16_nhwc.restype = i32
    L.sw_conv2d_bf16_nhwc.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [vp]
    L.sw_conv2d_f16_nhwc.restype = i32
    L.sw_conv2d_f16_nhwc.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [vp]
    L.sw_conv2d_s8_nhwc_requant.restype = i32
    L.sw_conv2d_s8_nhwc_requant.argtypes = [vp, vp, vp, vp, vp] + [i32] * 10 + [vp]
    L.sw_conv2d_s8_requant.restype = i32
    L.sw_conv2d_s8_requant.argtypes = [vp, vp, vp, vp, vp] + [i32] * 10 + [vp]
    L.sw_s8_packed_filter_bytes.restype = i64
    L.sw_s8_packed_filter_bytes.argtypes = [i32] * 4
    L.sw_s8_pack_filter.restype = i32
    L.sw_s8_pack_filter.argtypes = [vp, vp] + [i32] * 4 + [vp]
    L.sw_conv2d_s8_packed.restype = i32
    L.sw_conv2d_s8_packed.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.sw_conv2d_s8_packed_requant.restype = i32
    L.sw_conv2d_s8_packed_requant.argtypes = [vp, vp, vp, vp, vp] + [i32] * 10 + [vp]
    L.sw_probe.restype = i32
    L.sw_probe.argtypes = [i32, i32, vp]
    L.sw_probe_ops.restype = i64
    L.sw_probe_ops.argtypes = [i32, i32]
    L.sw_out_dim.restype = i64
    L.sw_out_dim.argtypes = [i64, i32, i32, i32]
    L.sw_out_dim_dilated.restype = i64
    L.sw_out_dim_dilated.argtypes = [i64, i32, i32, i32, i32]
    L.sw_last_kernel.restype = ctypes.c_char_p
    L.sw_last_kernel.argtypes = []
    L.sw_workspace_bytes.restype = ctypes.c_size_t
    L.sw_workspace_bytes.argtypes = []
    L.sw_status_string.restype = ctypes.c_char_p
    L.sw_status_string.argtypes = [i32]
    L.sw_version.restype = i32
    L.sw_version.argtypes = []
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().sw_status_string(int(status)).decode()


def sw_conv2d_s8_nhwc(x, w, stride: int = 1, pad: int = 0, bias=None, scale=None, relu: bool = False, out=None,
                      stream=None):
    """Channel-last int8 convolution: x [N,H,W,C_in] int8, w [C_out,R,S,C_in] int8 -> y [N,H_out,W_out,C_out]
    int32 (exact sums), or int8 when `scale` ([C_out] fp32, with optional int32 `bias`) is given:
    clamp(rne(scale * float(acc + bias)), 0 if relu else -128, 127)."""
    import torch

    N, H, W, C_in = x.shape
    C_out, R, S, C_in_w = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    rq = scale is not None
    name = "sw_conv2d_s8_nhwc_requant" if rq else "sw_conv2d_s8_nhwc"
    if out is None:
        out = torch.empty(_out_shape(name, N, sw_out_dim(H, R, stride, pad), sw_out_dim(W, S, stride, pad), C_out),
                          dtype=torch.int8 if rq else torch.int32, device=x.device)
    if rq:
        rc = lib().sw_conv2d_s8_nhwc_requant(_dev(x, torch.int8, 4, "x"), _dev(w, torch.int8, 4, "w"),
                                             _dev(bias, torch.int32, 1, "bias") if bias is not None else None,
                                             _dev(scale, torch.float32, 1, "scale"), _dev(out, torch.int8, 4, "y"),
                                             N, H, W, C_in, C_out, R, S, stride, pad, 1 if relu else 0,
                                             _stream(stream))
    else:
        rc = lib().sw_conv2d_s8_nhwc(_dev(x, torch.int8, 4, "x"), _dev(w, torch.int8, 4, "w"),
                                     _dev(out, torch.int32, 4, "y"), N, H, W, C_in, C_out, R, S, stride, pad,
                                     _stream(stream))
    _check(rc, name)
    return out


def sw_conv2d_nhwc(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False, out=None,
                   stream=None):
    """Channel-last convolution: x [N,H,W,C_in], w [C_out,R,S,C_in] -> y [N,H_out,W_out,C_out] = act(conv + bias[co]);
    fp32 tensors, or 16-bit tensors (torch.bfloat16 / torch.float16: fp32 accumulation, one rounding of the result);
    bias [C_out] fp32."""
    import torch

    N, H, W, C_in = x.shape
    C_out, R, S, C_in_w = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    dt = x.dtype if x.dtype in (torch.bfloat16, torch.float16) else torch.float32
    name = {torch.bfloat16: "sw_conv2d_bf16_nhwc", torch.float16: "sw_conv2d_f16_nhwc", torch.float32: "sw_conv2d_nhwc"}[dt]
    if out is None:
        out = torch.empty(_out_shape(name, N, sw_out_dim_dilated(H, R, stride, pad, dilation),
                                     sw_out_dim_dilated(W, S, stride, pad, dilation), C_out), dtype=dt, device=x.device)
    fn = getattr(lib(), name)
    rc = fn(_dev(x, dt, 4, "x"), _dev(w, dt, 4, "w"), _dev(bias, torch.float32, 1, "bias") if bias is not None else None,
            _dev(out, dt, 4, "y"), N, H, W, C_in, C_out, R, S, stride, pad, dilation, 1 if relu else 0, _stream(stream))
    _check(rc, name)
    return out


def sw_conv2d_bf16_nhwc(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False, out=None,
                        stream=None):
    """sw_conv2d_nhwc on torch.bfloat16 tensors (bf16 in and out, fp32 accumulation)."""
    import torch

    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16:
        raise TypeError("sw_conv2d_bf16_nhwc takes torch.bfloat16 tensors")
    return sw_conv2d_nhwc(x, w, stride, pad, dilation, bias, relu, out, stream)


def sw_conv2d_f16_nhwc(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, bias=None, relu: bool = False, out=None,
                       stream=None):
    """sw_conv2d_nhwc on torch.float16 tensors (half precision in and out, fp32 accumulation)."""
    import torch

    if x.dtype != torch.float16 or w.dtype != torch.float16:
        raise TypeError("sw_conv2d_f16_nhwc takes torch.float16 tensors")
    return sw_conv2d_nhwc(x, w, stride, pad, dilation, bias, relu, out, stream)


def sw_conv2d_s8_requant(x, w, bias, scale, stride: int = 1, pad: int = 0, relu: bool = False, out=None, stream=None):
    """x [N,C_in,H,W] int8, w [C_out,C_in,R,S] int8, bias [C_out] int32 or None, scale [C_out] fp32 ->
    y [N,C_out,H_out,W_out] int8 = clamp(rne(scale * float(acc + bias)), 0 if relu else -128, 127)."""
    import torch

    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_s8_requant", N, C_out, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.int8, device=x.device)
    b = _dev(bias, torch.int32, 1, "bias") if bias is not None else None
    rc = lib().sw_conv2d_s8_requant(_dev(x, torch.int8, 4, "x"), _dev(w, torch.int8, 4, "w"), b,
                                    _dev(scale, torch.float32, 1, "scale"), _dev(out, torch.int8, 4, "y"),
                                    N, C_in, C_out, H, W, R, S, stride, pad, 1 if relu else 0, _stream(stream))
    _check(rc, "sw_conv2d_s8_requant")
    return out


def sw_out_dim(n_in: int, k: int, stride: int, pad: int) -> int:
    return int(lib().sw_out_dim(n_in, k, stride, pad))


def sw_out_dim_dilated(n_in: int, k: int, stride: int, pad: int, dilation: int) -> int:
    return int(lib().sw_out_dim_dilated(n_in, k, stride, pad, dilation))


def sw_last_kernel() -> str:
    """Name (with template arguments) of the kernel the calling thread's most recent call enqueued."""
    return lib().sw_last_kernel().decode()


SW_PROBE_MFMA_F32, SW_PROBE_MFMA_I8, SW_PROBE_FMA_F32, SW_PROBE_FMA_MFMA_F32, SW_PROBE_MFMA_F32_FED, SW_PROBE_MFMA_F32_FED2, SW_PROBE_MFMA_BF16 = 0, 1, 2, 3, 4, 5, 6


def sw_probe(kind: int, iters: int, stream=None) -> int:
    """Enqueue the arithmetic-only probe kernel of `kind`; returns the number of operations it performs."""
    _check(lib().sw_probe(kind, iters, _stream(stream)), "sw_probe")
    return int(lib().sw_probe_ops(kind, iters))


def sw_workspace_bytes() -> int:
    return int(lib().sw_workspace_bytes())


def sw_version() -> int:
    return int(lib().sw_version())


def _stream(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t, dtype, ndim, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype or t.dim() != ndim or not t.is_contiguous():
        raise ValueError(f"{name}: expected contiguous {dtype} with {ndim} dims, got {t.dtype} {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _check(rc: int, what: str):
    if rc != SW_OK:
        raise SwError(rc, what)


def _out_shape(what, *dims):
    if min(dims) <= 0:
        raise SwError(SW_ERR_SHAPE, what)
    return dims


def sw_conv1d(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """x [rows, len] fp32, w [k] fp32 -> y [rows, len_out] fp32 (device tensors)."""
    import torch

    rows, length = x.shape
    k = w.shape[0]
    if out is None:
        out = torch.empty(_out_shape("sw_conv1d", rows, sw_out_dim(length, k, stride, pad)),
                          dtype=torch.float32, device=x.device)
    rc = lib().sw_conv1d(_dev(x, torch.float32, 2, "x"), _dev(w, torch.float32, 1, "w"),
                         _dev(out, torch.float32, 2, "y"), rows, length, k, stride, pad, _stream(stream))
    _check(rc, "sw_conv1d")
    return out


def sw_pool1d(x, window: int, stride: int = 1, mode: int = SW_POOL_AVG, out=None, stream=None):
    """x [rows, len] fp32 -> y [rows, len_out] fp32; mode SW_POOL_AVG or SW_POOL_MAX."""
    import torch

    rows, length = x.shape
    if out is None:
        out = torch.empty(_out_shape("sw_pool1d", rows, sw_out_dim(length, window, stride, 0)),
                          dtype=torch.float32, device=x.device)
    rc = lib().sw_pool1d(_dev(x, torch.float32, 2, "x"), _dev(out, torch.float32, 2, "y"), rows, length,
                         window, stride, mode, _stream(stream))
    _check(rc, "sw_pool1d")
    return out


def sw_pool2d(x, R: int, S: int, stride: int = 1, pad: int = 0, mode: int = SW_POOL_AVG, out=None, stream=None):
    """x [N,C,H,W] fp32 -> y [N,C,H_out,W_out] fp32; mode SW_POOL_AVG (divisor R*S) or SW_POOL_MAX."""
    import torch

    N, C, H, W = x.shape
    if out is None:
        out = torch.empty(_out_shape("sw_pool2d", N, C, sw_out_dim(H, R, stride, pad), sw_out_dim(W, S, stride, pad)),
                          dtype=torch.float32, device=x.device)
    rc = lib().sw_pool2d(_dev(x, torch.float32, 4, "x"), _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S,
                         stride, pad, mode, _stream(stream))
    _check(rc, "sw_pool2d")
    return out


def sw_conv2d(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """x [N,C_in,H,W] fp32, w [C_out,C_in,R,S] fp32 -> y [N,C_out,H_out,W_out] fp32."""
    import torch

    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d", N, C_out, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                         _dev(out, torch.float32, 4, "y"), N, C_in, C_out, H, W, R, S, stride, pad,
                         _stream(stream))
    _check(rc, "sw_conv2d")
    return out


def sw_conv2d_bias_relu(x, w, bias, stride: int = 1, pad: int = 0, relu: bool = False, out=None, stream=None):
    """x [N,C_in,H,W] fp32, w [C_out,C_in,R,S] fp32, bias [C_out] fp32 or None -> y = act(conv + bias)."""
    import torch

    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    if bias is not None and tuple(bias.shape) != (C_out,):
        raise ValueError("one bias per output channel")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_bias_relu", N, C_out, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_bias_relu(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                   _dev(bias, torch.float32, 1, "bias") if bias is not None else None,
                                   _dev(out, torch.float32, 4, "y"), N, C_in, C_out, H, W, R, S, stride, pad,
                                   1 if relu else 0, _stream(stream))
    _check(rc, "sw_conv2d_bias_relu")
    return out


def sw_conv2d_depthwise_bias_relu(x, w, bias, stride: int = 1, pad: int = 0, relu: bool = False, out=None, stream=None):
    """x [N,C,H,W] fp32, w [C,1,R,S] fp32, bias [C] fp32 or None -> y = act(depthwise conv + bias)."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if bias is not None and tuple(bias.shape) != (C,):
        raise ValueError("one bias per channel")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise_bias_relu", N, C, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_depthwise_bias_relu(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                             _dev(bias, torch.float32, 1, "bias") if bias is not None else None,
                                             _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S, stride, pad,
                                             1 if relu else 0, _stream(stream))
    _check(rc, "sw_conv2d_depthwise_bias_relu")
    return out


def sw_dw_pw_block(x, w_dw, b_dw, w_pw, b_pw, relu_dw: bool = True, relu_pw: bool = False, out=None, stream=None):
    """Depthwise 3x3 (stride 1, pad 1) + bias + rectifier, then pointwise 1x1 + bias + rectifier, in one launch:
    x [N,C,H,W], w_dw [C,1,3,3], b_dw [C] or None, w_pw [C_out,C,1,1], b_pw [C_out] or None -> y [N,C_out,H,W]."""
    import torch

    N, C, H, W = x.shape
    if tuple(w_dw.shape) != (C, 1, 3, 3):
        raise ValueError("depthwise weights must be [C,1,3,3]")
    C_out = w_pw.shape[0]
    if tuple(w_pw.shape) != (C_out, C, 1, 1):
        raise ValueError("pointwise weights must be [C_out,C,1,1]")
    if out is None:
        out = torch.empty((N, C_out, H, W), dtype=torch.float32, device=x.device)
    f32 = torch.float32
    rc = lib().sw_dw_pw_block(_dev(x, f32, 4, "x"), _dev(w_dw, f32, 4, "w_dw"),
                              _dev(b_dw, f32, 1, "b_dw") if b_dw is not None else None, _dev(w_pw, f32, 4, "w_pw"),
                              _dev(b_pw, f32, 1, "b_pw") if b_pw is not None else None, _dev(out, f32, 4, "y"),
                              N, C, C_out, H, W, 1 if relu_dw else 0, 1 if relu_pw else 0, _stream(stream))
    _check(rc, "sw_dw_pw_block")
    return out


def sw_conv2d_dilated(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, out=None, stream=None):
    """x [N,C_in,H,W] fp32, w [C_out,C_in,R,S] fp32, taps `dilation` positions apart -> y fp32."""
    import torch

    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_dilated", N, C_out, sw_out_dim_dilated(H, R, stride, pad, dilation),
                                     sw_out_dim_dilated(W, S, stride, pad, dilation)),
                          dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_dilated(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                 _dev(out, torch.float32, 4, "y"), N, C_in, C_out, H, W, R, S, stride, pad, dilation,
                                 _stream(stream))
    _check(rc, "sw_conv2d_dilated")
    return out


def sw_conv2d_depthwise_dilated(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, out=None, stream=None):
    """x [N,C,H,W] fp32, w [C,1,R,S] fp32, taps `dilation` positions apart -> y fp32."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise_dilated", N, C,
                                     sw_out_dim_dilated(H, R, stride, pad, dilation),
                                     sw_out_dim_dilated(W, S, stride, pad, dilation)),
                          dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_depthwise_dilated(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                           _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S, stride, pad,
                                           dilation, _stream(stream))
    _check(rc, "sw_conv2d_depthwise_dilated")
    return out


def sw_conv2d_depthwise(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """x [N,C,H,W] fp32, w [C,1,R,S] fp32 -> y [N,C,H_out,W_out] fp32."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise", N, C, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_depthwise(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                   _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S, stride, pad,
                                   _stream(stream))
    _check(rc, "sw_conv2d_depthwise")
    return out


def sw_conv2d_depthwise_bf16(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """x [N,C,H,W] bfloat16, w [C,1,R,S] fp32 -> y [N,C,H_out,W_out] bfloat16 (fp32 accumulation, one rounding)."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise_bf16", N, C, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.bfloat16, device=x.device)
    rc = lib().sw_conv2d_depthwise_bf16(_dev(x, torch.bfloat16, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                        _dev(out, torch.bfloat16, 4, "y"), N, C, H, W, R, S, stride, pad,
                                        _stream(stream))
    _check(rc, "sw_conv2d_depthwise_bf16")
    return out


def sw_conv2d_depthwise_jit(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """As sw_conv2d_depthwise, through the kernel generated at run time for this geometry (compiled on first use)."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise_jit", N, C, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_depthwise_jit(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                       _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S, stride, pad,
                                       _stream(stream))
    _check(rc, "sw_conv2d_depthwise_jit")
    return out


def sw_conv2d_depthwise_dilated_jit(x, w, stride: int = 1, pad: int = 0, dilation: int = 1, out=None, stream=None):
    """sw_conv2d_depthwise_dilated through a kernel generated at run time for the geometry (stride 1 or 2, any dilation)."""
    import torch

    N, C, H, W = x.shape
    Cw, one, R, S = w.shape
    if Cw != C or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_depthwise_dilated_jit", N, C, sw_out_dim_dilated(H, R, stride, pad, dilation),
                                     sw_out_dim_dilated(W, S, stride, pad, dilation)), dtype=torch.float32, device=x.device)
    rc = lib().sw_conv2d_depthwise_dilated_jit(_dev(x, torch.float32, 4, "x"), _dev(w, torch.float32, 4, "w"),
                                               _dev(out, torch.float32, 4, "y"), N, C, H, W, R, S, stride, pad, dilation,
                                               _stream(stream))
    _check(rc, "sw_conv2d_depthwise_dilated_jit")
    return out


def sw_jit_prepare_depthwise_dilated(H: int, W: int, R: int, S: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
    """Compile and load the generated kernel of a strided / dilated geometry ahead of its first use; a status code."""
    return int(lib().sw_jit_prepare_depthwise_dilated(H, W, R, S, stride, pad, dilation))


def sw_jit_compile_check_dilated(H: int, W: int, R: int, S: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
    """Compile only (no device needed): does the generated source build for the geometry?  A status code."""
    return int(lib().sw_jit_compile_check_dilated(H, W, R, S, stride, pad, dilation))


def sw_jit_prepare_depthwise(H: int, W: int, R: int, S: int, stride: int = 1, pad: int = 0) -> int:
    """Compile and load the generated kernel of a geometry; returns the status (SW_ERR_UNSUPPORTED: the
    precompiled kernels serve it)."""
    return int(lib().sw_jit_prepare_depthwise(H, W, R, S, stride, pad))


def sw_jit_compile_check(H: int, W: int, R: int, S: int, stride: int = 1, pad: int = 0) -> int:
    """Compile only (no device needed); returns the status."""
    return int(lib().sw_jit_compile_check(H, W, R, S, stride, pad))


def sw_jit_cached_kernels() -> int:
    return int(lib().sw_jit_cached_kernels())


def sw_conv2d_s8(x, w, stride: int = 1, pad: int = 0, out=None, stream=None):
    """x [N,C_in,H,W] int8, w [C_out,C_in,R,S] int8 -> y [N,C_out,H_out,W_out] int32 (exact sums)."""
    import torch

    N, C_in, H, W = x.shape
    C_out, C_in_w, R, S = w.shape
    if C_in_w != C_in:
        raise ValueError("channel mismatch between x and w")
    if out is None:
        out = torch.empty(_out_shape("sw_conv2d_s8", N, C_out, sw_out_dim(H, R, stride, pad),
                                     sw_out_dim(W, S, stride, pad)), dtype=torch.int32, device=x.device)
    rc = lib().sw_conv2d_s8(_dev(x, torch.int8, 4, "x"), _dev(w, torch.int8, 4, "w"),
                            _dev(out, torch.int32, 4, "y"), N, C_in, C_out, H, W, R, S, stride, pad,
                            _stream(stream))
    _check(rc, "sw_conv2d_s8")
    return out


def sw_s8_packed_filter_bytes(C_in: int, C_out: int, R: int, S: int) -> int:
    return int(lib().sw_s8_packed_filter_bytes(C_in, C_out, R, S))


def sw_s8_pack_filter(w, out=None, stream=None):
    """w [C_out,C_in,R,S] int8 -> the filters in the matrix instruction's operand order (1-D int8 tensor of
    sw_s8_packed_filter_bytes bytes), for sw_conv2d_s8_packed."""
    import torch

    C_out, C_in, R, S = w.shape
    nbytes = sw_s8_packed_filter_bytes(C_in, C_out, R, S)
    if nbytes <= 0:
        raise SwError(SW_ERR_SHAPE, "sw_s8_pack_filter")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.int8, device=w.device)
    rc = lib().sw_s8_pack_filter(_dev(w, torch.int8, 4, "w"), _dev(out, torch.int8, 1, "packed"), C_in, C_out, R, S,
                                 _stream(stream))
    _check(rc, "sw_s8_pack_filter")
    return out


def sw_conv2d_s8_packed(x, packed, C_out: int, R: int, S: int, stride: int = 1, pad: int = 0, bias=None, scale=None,
                        relu: bool = False, out=None, stream=None):
    """x [N,C_in,H,W] int8 and filters packed by sw_s8_pack_filter -> y [N,C_out,H_out,W_out] int32 (exact sums),
    or int8 when `scale` ([C_out] fp32, with optional int32 `bias`) is given, as sw_conv2d_s8_requant."""
    import torch

    N, C_in, H, W = x.shape
    rq = scale is not None
    name = "sw_conv2d_s8_packed_requant" if rq else "sw_conv2d_s8_packed"
    if out is None:
        out = torch.empty(_out_shape(name, N, C_out, sw_out_dim(H, R, stride, pad), sw_out_dim(W, S, stride, pad)),
                          dtype=torch.int8 if rq else torch.int32, device=x.device)
    if rq:
        rc = lib().sw_conv2d_s8_packed_requant(_dev(x, torch.int8, 4, "x"), _dev(packed, torch.int8, 1, "packed"),
                                               _dev(bias, torch.int32, 1, "bias") if bias is not None else None,
                                               _dev(scale, torch.float32, 1, "scale"), _dev(out, torch.int8, 4, "y"),
                                               N, C_in, C_out, H, W, R, S, stride, pad, 1 if relu else 0,
                                               _stream(stream))
    else:
        rc = lib().sw_conv2d_s8_packed(_dev(x, torch.int8, 4, "x"), _dev(packed, torch.int8, 1, "packed"),
                                       _dev(out, torch.int32, 4, "y"), N, C_in, C_out, H, W, R, S, stride, pad,
                                       _stream(stream))
    _check(rc, name)
    return out
