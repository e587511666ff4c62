"""numpy front end of the CPU oracle (oracle/vq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The HIP library and its Python binding never
import this package, and this package imports nothing of theirs.

Each function marshals numpy arrays to the C routine of the same name; all of the
arithmetic is in the C file, whose header states what each step follows in the
paper (Sec. 3.1 Eq. 2, Sec. 4.1, Sec. 4.2 Eq. 3, and the appendix on the hardware
implementation of quantized linear layers).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vq_oracle.c")
_LIB = os.path.join(_HERE, "libvq_oracle.so")
# A test may point this at another build of the same source (the sanitizer build of
# tests/test_sanitizers.py); it is then loaded as it is and never rebuilt here.
_LIB_OVERRIDE = os.environ.get("VQ_ORACLE_LIB")

# No fused multiply-add, no reassociation: every fp32 operation rounds on its own.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
          "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared library."""
    if _LIB_OVERRIDE:
        return _LIB_OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_half_to_float.restype = ctypes.c_float
        lib.oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.oracle_float_to_half.restype = ctypes.c_uint16
        lib.oracle_float_to_half.argtypes = [ctypes.c_float]
        lib.oracle_quantize_per_token.argtypes = [p, p, p, p, i64, i64]
        lib.oracle_quantize_rows_f32.argtypes = [p, p, p, p, i64, i64]
        lib.oracle_gelu.argtypes = [p, ci, p, i64, i64]
        lib.oracle_layernorm_modulate.argtypes = [p, p, p, i64, ctypes.c_double, p, i64, i64]
        lib.oracle_residual.argtypes = [p, p, p, i64, p, i64, i64]
        lib.oracle_channel_absmax_f16.argtypes = [p, p, i64, i64]
        lib.oracle_channel_absmax_f32.argtypes = [p, p, i64, i64]
        lib.oracle_balance_mask.argtypes = [p, p, ctypes.c_double, p, p, i64]
        lib.oracle_hadamard_rotate.argtypes = [p, p, i64, p, p, i64, i64]
        lib.oracle_rotate_weight.argtypes = [p, p, i64, p, p, i64, i64]
        lib.oracle_gemm_f16.argtypes = [p, p, p, p, i64, i64, i64]
        lib.oracle_quantize_static.argtypes = [p, p, ctypes.c_float, p, i64, i64]
        lib.oracle_quantize_weight.argtypes = [p, p, ci, p, p, i64, i64]
        lib.oracle_pack_int4.argtypes = [p, p, i64, i64]
        lib.oracle_unpack_int4.argtypes = [p, p, i64, i64]
        lib.oracle_gemm_i8.argtypes = [p, p, p, i64, i64, i64]
        lib.oracle_dequant.argtypes = [p, p, p, p, p, i64, i64]
        lib.oracle_linear.argtypes = [p, p, p, ci, p, p, p, p, p, p, p, i64, i64, i64]
        for name in ("oracle_channel_absmax_f16", "oracle_channel_absmax_f32", "oracle_balance_mask",
                     "oracle_hadamard_rotate", "oracle_rotate_weight", "oracle_gemm_f16", "oracle_quantize_static", "oracle_quantize_rows_f32", "oracle_gelu", "oracle_layernorm_modulate",
                     "oracle_residual",
                     "oracle_quantize_per_token", "oracle_quantize_weight", "oracle_pack_int4",
                     "oracle_unpack_int4", "oracle_gemm_i8", "oracle_dequant", "oracle_linear"):
            getattr(lib, name).restype = ci
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc: int, what: str) -> None:
    if rc == 2:
        raise OracleError(f"{what}: integer sum does not fit int32")
    if rc != 0:
        raise OracleError(f"{what}: bad argument (code {rc})")


def _arr(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f16(a):
    """fp16 array -> its uint16 bit patterns (a view, no conversion)."""
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("expected a float16 array")
    return a.view(np.uint16)


def half_to_float(bits: int) -> float:
    return float(_load().oracle_half_to_float(int(bits) & 0xFFFF))


def float_to_half(value) -> int:
    return int(_load().oracle_float_to_half(ctypes.c_float(float(np.float32(value)))))


def quantize_per_token(x_f16, chan_mul=None):
    """X fp16 [M,K], chan_mul fp32 [K] or None -> (xq int8 [M,K], x_scale fp32 [M])."""
    xb = _f16(x_f16)
    M, K = xb.shape
    cm = None if chan_mul is None else _arr(chan_mul, np.float32, (K,))
    xq = np.empty((M, K), np.int8)
    xs = np.empty((M,), np.float32)
    _check(_load().oracle_quantize_per_token(_ptr(xb), _ptr(cm), _ptr(xq), _ptr(xs), M, K),
           "quantize_per_token")
    return xq, xs


def quantize_rows_f32(t_f32, chan_mul=None):
    """The quantizer steps on rows that already are fp32: t [M,K] -> (xq, x_scale)."""
    t = _arr(t_f32, np.float32)
    M, K = t.shape
    cm = None if chan_mul is None else _arr(chan_mul, np.float32, (K,))
    xq = np.empty((M, K), np.int8)
    xs = np.empty((M,), np.float32)
    _check(_load().oracle_quantize_rows_f32(_ptr(t), _ptr(cm), _ptr(xq), _ptr(xs), M, K),
           "quantize_rows_f32")
    return xq, xs


def gelu(h_f16, approximate: bool = False):
    """GELU of fp16 [M,K] (exact, or the tanh form), evaluated in fp64 -> fp32 [M,K]."""
    hb = _f16(h_f16)
    M, K = hb.shape
    t = np.empty((M, K), np.float32)
    _check(_load().oracle_gelu(_ptr(hb), int(bool(approximate)), _ptr(t), M, K), "gelu")
    return t


def _per_sample(a, M, K, tokens_per_sample, what):
    if a is None:
        return None
    B = (M + tokens_per_sample - 1) // tokens_per_sample
    a = _arr(a, np.float32)
    if a.shape != (B, K):
        raise ValueError(f"{what}: expected shape {(B, K)}, got {a.shape}")
    return a


def layernorm_modulate(x_f16, scale=None, shift=None, tokens_per_sample=None, eps: float = 1e-6):
    """LayerNorm over the channels of each token, then (1 + scale[b]) * y + shift[b] with
    b = m // tokens_per_sample; fp64 -> fp32 [M,K]."""
    xb = _f16(x_f16)
    M, K = xb.shape
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    sc = _per_sample(scale, M, K, T, "scale")
    sh = _per_sample(shift, M, K, T, "shift")
    t = np.empty((M, K), np.float32)
    _check(_load().oracle_layernorm_modulate(_ptr(xb), _ptr(sc), _ptr(sh), T, float(eps), _ptr(t), M, K),
           "layernorm_modulate")
    return t


def residual(x_f16, y_f16, gate=None, tokens_per_sample=None):
    """r = x + gate[b] * y in fp32 (product and sum rounded), narrowed to fp16 [M,K]."""
    xb = _f16(x_f16)
    yb = _f16(y_f16)
    if xb.shape != yb.shape:
        raise ValueError("x and y differ in shape")
    M, K = xb.shape
    T = int(tokens_per_sample) if tokens_per_sample else max(M, 1)
    g = _per_sample(gate, M, K, T, "gate")
    r = np.empty((M, K), np.uint16)
    _check(_load().oracle_residual(_ptr(xb), _ptr(yb), _ptr(g), T, _ptr(r), M, K), "residual")
    return r.view(np.float16)


def gelu_quantize(h_f16, chan_mul=None, approximate: bool = False):
    """GELU fused with the quantizer: returns (t fp32, xq, x_scale)."""
    t = gelu(h_f16, approximate)
    return (t,) + quantize_rows_f32(t, chan_mul)


def layernorm_quantize(x_f16, scale=None, shift=None, tokens_per_sample=None, eps: float = 1e-6,
                       chan_mul=None):
    """LayerNorm + modulation fused with the quantizer: returns (t fp32, xq, x_scale)."""
    t = layernorm_modulate(x_f16, scale, shift, tokens_per_sample, eps)
    return (t,) + quantize_rows_f32(t, chan_mul)


def residual_quantize(x_f16, y_f16, gate=None, tokens_per_sample=None, chan_mul=None):
    """Residual add fused with the quantizer: returns (r fp16, xq, x_scale)."""
    r = residual(x_f16, y_f16, gate, tokens_per_sample)
    return (r,) + quantize_per_token(r, chan_mul)


def channel_absmax(a):
    """max over the rows of |a| per column: fp16 activations [M,K] or fp32 weights [N,K] -> fp32 [K]."""
    a = np.ascontiguousarray(a)
    R, K = a.shape
    out = np.empty((K,), np.float32)
    if a.dtype == np.float16:
        _check(_load().oracle_channel_absmax_f16(_ptr(a.view(np.uint16)), _ptr(out), R, K), "channel_absmax")
    elif a.dtype == np.float32:
        _check(_load().oracle_channel_absmax_f32(_ptr(a), _ptr(out), R, K), "channel_absmax")
    else:
        raise TypeError("expected float16 or float32")
    return out


def balance_mask(amax_x, amax_w, alpha: float):
    """Eq. 3: s = amax_x^alpha / amax_w^(1 - alpha) -> (s fp32 [K], chan_mul = 1/s fp32 [K])."""
    ax = _arr(amax_x, np.float32)
    K = ax.shape[0]
    aw = _arr(amax_w, np.float32, (K,))
    s = np.empty((K,), np.float32)
    cm = np.empty((K,), np.float32)
    _check(_load().oracle_balance_mask(_ptr(ax), _ptr(aw), float(alpha), _ptr(s), _ptr(cm), K), "balance_mask")
    return s, cm


HADAMARD_BLOCK = 128


def hadamard_rotate(x_f16, chan_mul=None, block: int = HADAMARD_BLOCK):
    """(X * chan_mul) Q with Q block diagonal, blocks H_block / sqrt(block): fp16 [M,K] -> fp32 [M,K]."""
    xb = _f16(x_f16)
    M, K = xb.shape
    cm = None if chan_mul is None else _arr(chan_mul, np.float32, (K,))
    t = np.empty((M, K), np.float32)
    scratch = np.empty((M, K), np.float64)
    _check(_load().oracle_hadamard_rotate(_ptr(xb), _ptr(cm), int(block), _ptr(t), _ptr(scratch), M, K),
           "hadamard_rotate")
    return t


def rotate_weight(w_f32, chan_s=None, block: int = HADAMARD_BLOCK):
    """(W * s) Q, the weight side of the same rotation: fp32 [N,K] -> fp32 [N,K]."""
    w = _arr(w_f32, np.float32)
    N, K = w.shape
    s = None if chan_s is None else _arr(chan_s, np.float32, (K,))
    out = np.empty((N, K), np.float32)
    scratch = np.empty((N, K), np.float64)
    _check(_load().oracle_rotate_weight(_ptr(w), _ptr(s), int(block), _ptr(out), _ptr(scratch), N, K),
           "rotate_weight")
    return out


def hadamard_quantize(x_f16, chan_mul=None, block: int = HADAMARD_BLOCK):
    """Scaling, rotation, per-token quantization: returns (t fp32, xq, x_scale)."""
    t = hadamard_rotate(x_f16, chan_mul, block)
    return (t,) + quantize_rows_f32(t, None)


def gemm_f16(x_f16, w_f16, bias_f16=None):
    """FP16 linear layer: X fp16 [M,K], W fp16 [N,K] -> fp16 [M,N], summed in fp64."""
    xb, wb = _f16(x_f16), _f16(w_f16)
    M, K = xb.shape
    N = wb.shape[0]
    if wb.shape != (N, K):
        raise ValueError("weight shape")
    b = None if bias_f16 is None else _f16(bias_f16)
    y = np.empty((M, N), np.uint16)
    _check(_load().oracle_gemm_f16(_ptr(xb), _ptr(wb), _ptr(b), _ptr(y), M, N, K), "gemm_f16")
    return y.view(np.float16)


def quantize_static(x_f16, scale: float, chan_mul=None):
    """One fixed scale for the whole tensor: X fp16 [M,K] -> xq int8 [M,K], clipped at +-127."""
    xb = _f16(x_f16)
    M, K = xb.shape
    cm = None if chan_mul is None else _arr(chan_mul, np.float32, (K,))
    xq = np.empty((M, K), np.int8)
    _check(_load().oracle_quantize_static(_ptr(xb), _ptr(cm), ctypes.c_float(float(np.float32(scale))),
                                          _ptr(xq), M, K), "quantize_static")
    return xq


def quantize_weight(w_f32, chan_s=None, bits: int = 8):
    """W fp32 [N,K], s fp32 [K] or None -> (wq int8 [N,K] in [-qmax,qmax], w_scale fp32 [N])."""
    w = _arr(w_f32, np.float32)
    N, K = w.shape
    s = None if chan_s is None else _arr(chan_s, np.float32, (K,))
    wq = np.empty((N, K), np.int8)
    ws = np.empty((N,), np.float32)
    _check(_load().oracle_quantize_weight(_ptr(w), _ptr(s), int(bits), _ptr(wq), _ptr(ws), N, K),
           "quantize_weight")
    return wq, ws


def pack_int4(wq):
    wq = _arr(wq, np.int8)
    N, K = wq.shape
    out = np.empty((N, K // 2), np.uint8)
    _check(_load().oracle_pack_int4(_ptr(wq), _ptr(out), N, K), "pack_int4")
    return out


def unpack_int4(packed):
    packed = _arr(packed, np.uint8)
    N, K2 = packed.shape
    out = np.empty((N, 2 * K2), np.int8)
    _check(_load().oracle_unpack_int4(_ptr(packed), _ptr(out), N, 2 * K2), "unpack_int4")
    return out


def gemm_i8(xq, wq):
    """xq int8 [M,K], wq int8 [N,K] -> acc int32 [M,N] (sum over K, checked in int64)."""
    xq = _arr(xq, np.int8)
    wq = _arr(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    acc = np.empty((M, N), np.int32)
    _check(_load().oracle_gemm_i8(_ptr(xq), _ptr(wq), _ptr(acc), M, N, K), "gemm_i8")
    return acc


def dequant(acc, x_scale, w_scale, bias_f16=None):
    """acc int32 [M,N] -> Y fp16 [M,N] = fp16(acc * x_scale[m] * w_scale[n] + bias[n])."""
    acc = _arr(acc, np.int32)
    M, N = acc.shape
    xs = _arr(x_scale, np.float32, (M,))
    ws = _arr(w_scale, np.float32, (N,))
    b = None if bias_f16 is None else _f16(bias_f16)
    if b is not None and b.shape != (N,):
        raise ValueError("bias shape")
    y = np.empty((M, N), np.uint16)
    _check(_load().oracle_dequant(_ptr(acc), _ptr(xs), _ptr(ws), _ptr(b), _ptr(y), M, N), "dequant")
    return y.view(np.float16)


def linear(x_f16, chan_mul, w, w_bits, w_scale, bias_f16=None):
    """The whole layer.  Returns a dict with y (fp16), xq, x_scale, acc."""
    xb = _f16(x_f16)
    M, K = xb.shape
    if w_bits == 8:
        wa = _arr(w, np.int8)
        N = wa.shape[0]
        if wa.shape != (N, K):
            raise ValueError("weight shape")
        scratch = None
    elif w_bits == 4:
        wa = _arr(w, np.uint8)
        N = wa.shape[0]
        if wa.shape != (N, K // 2) or K % 2:
            raise ValueError("packed weight shape")
        scratch = np.empty((N, K), np.int8)
    else:
        raise ValueError("w_bits must be 8 or 4")
    cm = None if chan_mul is None else _arr(chan_mul, np.float32, (K,))
    ws = _arr(w_scale, np.float32, (N,))
    b = None if bias_f16 is None else _f16(bias_f16)
    y = np.empty((M, N), np.uint16)
    xq = np.empty((M, K), np.int8)
    xs = np.empty((M,), np.float32)
    acc = np.empty((M, N), np.int32)
    _check(_load().oracle_linear(_ptr(xb), _ptr(cm), _ptr(wa), int(w_bits), _ptr(ws), _ptr(b),
                                 _ptr(y), _ptr(xq), _ptr(xs), _ptr(acc), _ptr(scratch), M, N, K),
           "linear")
    return {"y": y.view(np.float16), "xq": xq, "x_scale": xs, "acc": acc}


def num_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS, else the visible cores)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1
