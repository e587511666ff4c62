"""Thin Python binding of the C-ABI library libvidiq.so (declared in include/vq.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the quantized linear layer runs in the library's kernels.
There is no fallback: if the library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
# the in-tree build; VQ_LIBVIDIQ_PATH names another build of the same sources (e.g. one with host sanitizers)
LIB_PATH = os.environ.get("VQ_LIBVIDIQ_PATH") or os.path.join(PKG_DIR, "libvidiq.so")

VQ_OK = 0
STATUS_NAMES = {0: "VQ_OK", 1: "VQ_ERR_NULL", 2: "VQ_ERR_SHAPE", 3: "VQ_ERR_ALIGN",
                4: "VQ_ERR_WORKSPACE", 5: "VQ_ERR_LAUNCH", 6: "VQ_ERR_ARCH", 7: "VQ_ERR_BITS"}

# name -> (restype, argtypes); mirrors include/vq.h
_P, _I, _SZ = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
SIGNATURES = {
    "vq_quantize_per_token": (_I, [_P, _P, _P, _P, _I, _I, _P]),
    "vq_gelu_quantize": (_I, [_P, _I, _P, _P, _P, _I, _I, _P]),
    "vq_layernorm_quantize": (_I, [_P, _P, _P, _I, ctypes.c_float, _P, _P, _P, _I, _I, _P]),
    "vq_residual_quantize": (_I, [_P, _P, _P, _I, _P, _P, _P, _P, _I, _I, _P]),
    "vq_channel_absmax": (_I, [_P, _I, _P, _I, _I, _I, _P]),
    "vq_balance_mask": (_I, [_P, _P, ctypes.c_float, _P, _P, _I, _P]),
    "vq_hadamard_quantize": (_I, [_P, _P, _P, _P, _I, _I, _P]),
    "vq_rotate_weight": (_I, [_P, _P, _P, _I, _I, _P]),
    "vq_gemm_f16": (_I, [_P, _P, _P, _P, _I, _I, _I, _P]),
    "vq_quantize_static": (_I, [_P, _P, ctypes.c_float, _P, _I, _I, _P]),
    "vq_gemm_w8a8": (_I, [_P, _P, _P, _P, _P, _P, _P, _I, _I, _I, _P]),
    "vq_gemm_w4a8": (_I, [_P, _P, _P, _P, _P, _P, _P, _I, _I, _I, _P]),
    "vq_linear": (_I, [_P, _P, _P, _I, _P, _P, _P, _P, _SZ, _I, _I, _I, _P]),
    "vq_linear_workspace_bytes": (_SZ, [_I, _I, _I, _I]),
    "vq_layernorm_linear": (_I, [_P, _P, _P, _I, ctypes.c_float, _P, _P, _I, _P, _P, _P, _P, _SZ, _I, _I, _I, _P]),
    "vq_gelu_linear": (_I, [_P, _I, _P, _P, _I, _P, _P, _P, _P, _SZ, _I, _I, _I, _P]),
    "vq_residual_linear": (_I, [_P, _P, _P, _I, _P, _P, _P, _I, _P, _P, _P, _P, _SZ, _I, _I, _I, _P]),
    "vq_hadamard_linear": (_I, [_P, _P, _P, _I, _P, _P, _P, _P, _SZ, _I, _I, _I, _P]),
    "vq_linear_static": (_I, [_P, _P, _P, _I, _P, _P, _P, _I, _I, _I, _P]),
    "vq_quantize_weight": (_I, [_P, _P, _I, _P, _P, _I, _I, _P]),
    "vq_status_string": (ctypes.c_char_p, [_I]),
}


class VqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libvidiq.so; raises if it has not been built (python -m paper_2406_02540_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} not found: build it with `python -m paper_2406_02540_amd.build`")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def status_string(status: int) -> str:
    return lib().vq_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != VQ_OK:
        raise VqError(status, where)


def _dev(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous (dense row-major)")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def vq_quantize_per_token(x, chan_mul=None, xq=None, x_scale=None, stream=None):
    """x fp16 [M,K] (+ chan_mul fp32 [K]) -> (xq int8 [M,K], x_scale fp32 [M])."""
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    chan_mul = _dev(chan_mul, torch.float32, "chan_mul")
    if chan_mul is not None and tuple(chan_mul.shape) != (K,):
        raise ValueError("chan_mul must have shape [K]")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if x_scale is None:
        x_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _dev(xq, torch.int8, "xq"), _dev(x_scale, torch.float32, "x_scale")
    if tuple(xq.shape) != (M, K) or tuple(x_scale.shape) != (M,):
        raise ValueError("output shapes")
    _check(lib().vq_quantize_per_token(_ptr(x), _ptr(chan_mul), _ptr(xq), _ptr(x_scale), M, K,
                                       _stream(stream)), "vq_quantize_per_token")
    return xq, x_scale


def _quant_outputs(x, chan_mul, xq, x_scale):
    M, K = x.shape
    chan_mul = _dev(chan_mul, torch.float32, "chan_mul")
    if chan_mul is not None and tuple(chan_mul.shape) != (K,):
        raise ValueError("chan_mul must have shape [K]")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if x_scale is None:
        x_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _dev(xq, torch.int8, "xq"), _dev(x_scale, torch.float32, "x_scale")
    if tuple(xq.shape) != (M, K) or tuple(x_scale.shape) != (M,):
        raise ValueError("output shapes")
    return chan_mul, xq, x_scale


def _per_sample(t, M, K, tokens_per_sample, name):
    t = _dev(t, torch.float32, name)
    if t is not None and tuple(t.shape) != ((M + tokens_per_sample - 1) // tokens_per_sample, K):
        raise ValueError(f"{name} must have shape [ceil(M / tokens_per_sample), K]")
    return t


def vq_gelu_quantize(h, approximate=False, chan_mul=None, xq=None, x_scale=None, stream=None):
    """GELU (exact or tanh form) fused with the quantizer: h fp16 [M,K] -> (xq, x_scale)."""
    h = _dev(h, torch.float16, "h")
    M, K = h.shape
    chan_mul, xq, x_scale = _quant_outputs(h, chan_mul, xq, x_scale)
    _check(lib().vq_gelu_quantize(_ptr(h), int(bool(approximate)), _ptr(chan_mul), _ptr(xq), _ptr(x_scale),
                                  M, K, _stream(stream)), "vq_gelu_quantize")
    return xq, x_scale


def vq_layernorm_quantize(x, mod_scale=None, mod_shift=None, tokens_per_sample=None, eps=1e-6,
                          chan_mul=None, xq=None, x_scale=None, stream=None):
    """LayerNorm + (1 + scale) y + shift fused with the quantizer: x fp16 [M,K] -> (xq, x_scale)."""
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    mod_scale = _per_sample(mod_scale, M, K, T, "mod_scale")
    mod_shift = _per_sample(mod_shift, M, K, T, "mod_shift")
    chan_mul, xq, x_scale = _quant_outputs(x, chan_mul, xq, x_scale)
    _check(lib().vq_layernorm_quantize(_ptr(x), _ptr(mod_scale), _ptr(mod_shift), T, float(eps),
                                       _ptr(chan_mul), _ptr(xq), _ptr(x_scale), M, K, _stream(stream)),
           "vq_layernorm_quantize")
    return xq, x_scale


def vq_residual_quantize(x, y, gate=None, tokens_per_sample=None, r=None, chan_mul=None, xq=None,
                         x_scale=None, stream=None):
    """r = x + gate * y fused with the quantizer: fp16 [M,K] twice -> (r fp16, xq, x_scale)."""
    x = _dev(x, torch.float16, "x")
    y = _dev(y, torch.float16, "y")
    if y is None or tuple(y.shape) != tuple(x.shape):
        raise ValueError("y must have the shape of x")
    M, K = x.shape
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    gate = _per_sample(gate, M, K, T, "gate")
    if r is None:
        r = torch.empty((M, K), dtype=torch.float16, device=x.device)
    _dev(r, torch.float16, "r")
    if tuple(r.shape) != (M, K):
        raise ValueError("r must have the shape of x")
    chan_mul, xq, x_scale = _quant_outputs(x, chan_mul, xq, x_scale)
    _check(lib().vq_residual_quantize(_ptr(x), _ptr(y), _ptr(gate), T, _ptr(r), _ptr(chan_mul), _ptr(xq),
                                      _ptr(x_scale), M, K, _stream(stream)), "vq_residual_quantize")
    return r, xq, x_scale


def vq_channel_absmax(a, amax=None, accumulate=False, stream=None):
    """Per-column absmax of fp16 activations [M,K] or fp32 weights [N,K] -> amax fp32 [K]."""
    if not isinstance(a, torch.Tensor) or a.dtype not in (torch.float16, torch.float32):
        raise TypeError("a: expected a float16 or float32 device tensor")
    a = _dev(a, a.dtype, "a")
    R, K = a.shape
    if amax is None:
        if accumulate:
            raise ValueError("accumulate needs the running amax")
        amax = torch.empty((K,), dtype=torch.float32, device=a.device)
    _dev(amax, torch.float32, "amax")
    if tuple(amax.shape) != (K,):
        raise ValueError("amax must have shape [K]")
    _check(lib().vq_channel_absmax(_ptr(a), int(a.dtype == torch.float32), _ptr(amax), R, K, int(bool(accumulate)),
                                   _stream(stream)), "vq_channel_absmax")
    return amax


def vq_balance_mask(amax_x, amax_w, alpha, stream=None):
    """Eq. 3: (s, chan_mul = 1/s), fp32 [K] each, from the two absmax statistics."""
    amax_x = _dev(amax_x, torch.float32, "amax_x")
    amax_w = _dev(amax_w, torch.float32, "amax_w")
    K = amax_x.shape[0]
    if tuple(amax_x.shape) != (K,) or tuple(amax_w.shape) != (K,):
        raise ValueError("statistics must have shape [K]")
    s = torch.empty((K,), dtype=torch.float32, device=amax_x.device)
    cm = torch.empty_like(s)
    _check(lib().vq_balance_mask(_ptr(amax_x), _ptr(amax_w), float(alpha), _ptr(s), _ptr(cm), K, _stream(stream)),
           "vq_balance_mask")
    return s, cm


def vq_hadamard_quantize(x, chan_mul=None, xq=None, x_scale=None, stream=None):
    """Scaling, block Hadamard rotation, per-token quantizer: x fp16 [M,K] -> (xq, x_scale)."""
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    chan_mul, xq, x_scale = _quant_outputs(x, chan_mul, xq, x_scale)
    _check(lib().vq_hadamard_quantize(_ptr(x), _ptr(chan_mul), _ptr(xq), _ptr(x_scale), M, K, _stream(stream)),
           "vq_hadamard_quantize")
    return xq, x_scale


def vq_rotate_weight(w, chan_s=None, out=None, stream=None):
    """Weight side of the rotation: w fp32 [N,K] (* chan_s) -> fp32 [N,K]."""
    w = _dev(w, torch.float32, "w")
    N, K = w.shape
    chan_s = _dev(chan_s, torch.float32, "chan_s")
    if chan_s is not None and tuple(chan_s.shape) != (K,):
        raise ValueError("chan_s must have shape [K]")
    if out is None:
        out = torch.empty_like(w)
    _dev(out, torch.float32, "out")
    if tuple(out.shape) != (N, K):
        raise ValueError("out must have the shape of w")
    _check(lib().vq_rotate_weight(_ptr(w), _ptr(chan_s), _ptr(out), N, K, _stream(stream)), "vq_rotate_weight")
    return out


def vq_gemm_f16(x, w, bias=None, y=None, stream=None):
    """FP16 comparison layer: x fp16 [M,K], w fp16 [N,K] (+ bias fp16 [N]) -> y fp16 [M,N]."""
    x = _dev(x, torch.float16, "x")
    w = _dev(w, torch.float16, "w")
    M, K = x.shape
    N = w.shape[0]
    if tuple(w.shape) != (N, K):
        raise ValueError("weight shape does not match K")
    bias = _dev(bias, torch.float16, "bias")
    if bias is not None and tuple(bias.shape) != (N,):
        raise ValueError("bias must have shape [N]")
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    if tuple(y.shape) != (M, N):
        raise ValueError("y must have shape [M,N]")
    _check(lib().vq_gemm_f16(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), M, N, K, _stream(stream)), "vq_gemm_f16")
    return y


def vq_quantize_static(x, scale, chan_mul=None, xq=None, stream=None):
    """One fixed scale for the whole tensor: x fp16 [M,K] -> xq int8 [M,K] (clipped at +-127)."""
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    chan_mul = _dev(chan_mul, torch.float32, "chan_mul")
    if chan_mul is not None and tuple(chan_mul.shape) != (K,):
        raise ValueError("chan_mul must have shape [K]")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _dev(xq, torch.int8, "xq")
    if tuple(xq.shape) != (M, K):
        raise ValueError("xq must have shape [M,K]")
    _check(lib().vq_quantize_static(_ptr(x), _ptr(chan_mul), float(scale), _ptr(xq), M, K, _stream(stream)),
           "vq_quantize_static")
    return xq


def _gemm(fn_name, xq, x_scale, w, w_cols_div, w_dtype, w_scale, bias, y, want_acc, stream):
    xq = _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    w = _dev(w, w_dtype, "w")
    N = w.shape[0]
    if tuple(w.shape) != (N, K // w_cols_div) or K % w_cols_div:
        raise ValueError("weight shape does not match K")
    x_scale = _dev(x_scale, torch.float32, "x_scale")
    w_scale = _dev(w_scale, torch.float32, "w_scale")
    bias = _dev(bias, torch.float16, "bias")
    if tuple(x_scale.shape) != (M,) or tuple(w_scale.shape) != (N,) or \
            (bias is not None and tuple(bias.shape) != (N,)):
        raise ValueError("scale / bias shapes")
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _dev(y, torch.float16, "y")
    if tuple(y.shape) != (M, N):
        raise ValueError("y shape")
    acc = torch.empty((M, N), dtype=torch.int32, device=xq.device) if want_acc else None
    _check(getattr(lib(), fn_name)(_ptr(xq), _ptr(x_scale), _ptr(w), _ptr(w_scale), _ptr(bias),
                                   _ptr(y), _ptr(acc), M, N, K, _stream(stream)), fn_name)
    return (y, acc) if want_acc else y


def vq_gemm_w8a8(xq, x_scale, wq, w_scale, bias=None, y=None, return_acc=False, stream=None):
    """int8 [M,K] x int8 [N,K] -> fp16 [M,N] (and the int32 sums if return_acc)."""
    return _gemm("vq_gemm_w8a8", xq, x_scale, wq, 1, torch.int8, w_scale, bias, y, return_acc, stream)


def vq_gemm_w4a8(xq, x_scale, wq4, w_scale, bias=None, y=None, return_acc=False, stream=None):
    """int8 [M,K] x packed 4-bit [N,K/2] -> fp16 [M,N] (and the int32 sums if return_acc)."""
    return _gemm("vq_gemm_w4a8", xq, x_scale, wq4, 2, torch.uint8, w_scale, bias, y, return_acc,
                 stream)


def vq_linear_workspace_bytes(M, N, K, w_bits) -> int:
    return int(lib().vq_linear_workspace_bytes(int(M), int(N), int(K), int(w_bits)))


LINEAR_STATIC_SCRATCH_BYTES = 40 << 20  # VQ_LINEAR_STATIC_SCRATCH_BYTES of include/vq.h


def _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y, where):
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    if w_bits == 8:
        w = _dev(w, torch.int8, "w")
        ok = tuple(w.shape[1:]) == (K,)
    elif w_bits == 4:
        w = _dev(w, torch.uint8, "w")
        ok = K % 2 == 0 and tuple(w.shape[1:]) == (K // 2,)
    else:
        raise VqError(7, where)
    if not ok:
        raise ValueError("weight shape does not match K")
    N = w.shape[0]
    chan_mul = _dev(chan_mul, torch.float32, "chan_mul")
    w_scale = _dev(w_scale, torch.float32, "w_scale")
    bias = _dev(bias, torch.float16, "bias")
    if (chan_mul is not None and tuple(chan_mul.shape) != (K,)) or tuple(w_scale.shape) != (N,) \
            or (bias is not None and tuple(bias.shape) != (N,)):
        raise ValueError("chan_mul / scale / bias shapes")
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    if tuple(y.shape) != (M, N):
        raise ValueError("y shape")
    return x, chan_mul, w, w_scale, bias, y, M, N, K


def vq_linear_static(x, chan_mul, w, w_bits, w_scale, bias=None, y=None, stream=None):
    """The whole layer with the library's built-in scratch instead of a workspace (the call allocates nothing
    when y is given); layers whose int8 activations exceed LINEAR_STATIC_SCRATCH_BYTES raise VQ_ERR_WORKSPACE."""
    x, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y,
                                                             "vq_linear_static")
    _check(lib().vq_linear_static(_ptr(x), _ptr(chan_mul), _ptr(w), int(w_bits), _ptr(w_scale), _ptr(bias),
                                  _ptr(y), M, N, K, _stream(stream)), "vq_linear_static")
    return y


def _workspace(workspace, x, M, N, K, w_bits):
    if workspace is None:
        need = vq_linear_workspace_bytes(M, N, K, w_bits)
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=x.device)
    return _dev(workspace, torch.uint8, "workspace")


def vq_linear(x, chan_mul, w, w_bits, w_scale, bias=None, y=None, workspace=None, stream=None):
    """The whole layer on fp16 activations; workspace is a uint8 device tensor (allocated if None)."""
    x, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y, "vq_linear")
    workspace = _workspace(workspace, x, M, N, K, w_bits)
    _check(lib().vq_linear(_ptr(x), _ptr(chan_mul), _ptr(w), int(w_bits), _ptr(w_scale), _ptr(bias),
                           _ptr(y), _ptr(workspace), workspace.numel(), M, N, K, _stream(stream)),
           "vq_linear")
    return y


def vq_layernorm_linear(x, w, w_bits, w_scale, mod_scale=None, mod_shift=None, tokens_per_sample=None, eps=1e-6,
                        chan_mul=None, bias=None, y=None, workspace=None, stream=None):
    """LayerNorm + modulation, quantizer and GEMM in one call: x fp16 [M,K] -> y fp16 [M,N]."""
    x, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y,
                                                             "vq_layernorm_linear")
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    mod_scale = _per_sample(mod_scale, M, K, T, "mod_scale")
    mod_shift = _per_sample(mod_shift, M, K, T, "mod_shift")
    workspace = _workspace(workspace, x, M, N, K, w_bits)
    _check(lib().vq_layernorm_linear(_ptr(x), _ptr(mod_scale), _ptr(mod_shift), T, float(eps), _ptr(chan_mul),
                                     _ptr(w), int(w_bits), _ptr(w_scale), _ptr(bias), _ptr(y), _ptr(workspace),
                                     workspace.numel(), M, N, K, _stream(stream)), "vq_layernorm_linear")
    return y


def vq_gelu_linear(h, w, w_bits, w_scale, approximate=False, chan_mul=None, bias=None, y=None, workspace=None,
                   stream=None):
    """GELU, quantizer and GEMM in one call: h fp16 [M,K] -> y fp16 [M,N]."""
    h, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(h, chan_mul, w, w_bits, w_scale, bias, y,
                                                             "vq_gelu_linear")
    workspace = _workspace(workspace, h, M, N, K, w_bits)
    _check(lib().vq_gelu_linear(_ptr(h), int(bool(approximate)), _ptr(chan_mul), _ptr(w), int(w_bits),
                                _ptr(w_scale), _ptr(bias), _ptr(y), _ptr(workspace), workspace.numel(), M, N, K,
                                _stream(stream)), "vq_gelu_linear")
    return y


def vq_residual_linear(x, y_in, w, w_bits, w_scale, gate=None, tokens_per_sample=None, r=None, chan_mul=None,
                       bias=None, y=None, workspace=None, stream=None):
    """r = x + gate * y_in, quantizer and GEMM in one call: fp16 [M,K] twice -> (r fp16 [M,K], y fp16 [M,N])."""
    x, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y,
                                                             "vq_residual_linear")
    y_in = _dev(y_in, torch.float16, "y_in")
    if y_in is None or tuple(y_in.shape) != (M, K):
        raise ValueError("y_in must have the shape of x")
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    gate = _per_sample(gate, M, K, T, "gate")
    if r is None:
        r = torch.empty((M, K), dtype=torch.float16, device=x.device)
    _dev(r, torch.float16, "r")
    if tuple(r.shape) != (M, K):
        raise ValueError("r must have the shape of x")
    workspace = _workspace(workspace, x, M, N, K, w_bits)
    _check(lib().vq_residual_linear(_ptr(x), _ptr(y_in), _ptr(gate), T, _ptr(r), _ptr(chan_mul), _ptr(w),
                                    int(w_bits), _ptr(w_scale), _ptr(bias), _ptr(y), _ptr(workspace),
                                    workspace.numel(), M, N, K, _stream(stream)), "vq_residual_linear")
    return r, y


def vq_hadamard_linear(x, chan_mul, w, w_bits, w_scale, bias=None, y=None, workspace=None, stream=None):
    """Scaling, block Hadamard rotation, quantizer and GEMM in one call (w quantized from rotated weights)."""
    x, chan_mul, w, w_scale, bias, y, M, N, K = _linear_args(x, chan_mul, w, w_bits, w_scale, bias, y,
                                                             "vq_hadamard_linear")
    workspace = _workspace(workspace, x, M, N, K, w_bits)
    _check(lib().vq_hadamard_linear(_ptr(x), _ptr(chan_mul), _ptr(w), int(w_bits), _ptr(w_scale), _ptr(bias),
                                    _ptr(y), _ptr(workspace), workspace.numel(), M, N, K, _stream(stream)),
           "vq_hadamard_linear")
    return y


def vq_quantize_weight(w_f32, chan_s=None, w_bits=8, stream=None):
    """W fp32 [N,K] (+ s fp32 [K]) -> (wq int8 [N,K] or packed uint8 [N,K/2], w_scale fp32 [N])."""
    w_f32 = _dev(w_f32, torch.float32, "w")
    N, K = w_f32.shape
    chan_s = _dev(chan_s, torch.float32, "chan_s")
    if chan_s is not None and tuple(chan_s.shape) != (K,):
        raise ValueError("chan_s must have shape [K]")
    if w_bits == 8:
        wq = torch.empty((N, K), dtype=torch.int8, device=w_f32.device)
    elif w_bits == 4:
        wq = torch.empty((N, K // 2), dtype=torch.uint8, device=w_f32.device)
    else:
        raise VqError(7, "vq_quantize_weight")
    ws = torch.empty((N,), dtype=torch.float32, device=w_f32.device)
    _check(lib().vq_quantize_weight(_ptr(w_f32), _ptr(chan_s), int(w_bits), _ptr(wq), _ptr(ws), N, K,
                                    _stream(stream)), "vq_quantize_weight")
    return wq, ws
