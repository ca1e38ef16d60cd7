"""ctypes front-end of the CPU oracle (``sqp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports it and it
imports nothing from the product.  Arrays are numpy; fp16 travels as
``np.float16`` (viewed as ``uint16`` at the C boundary).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sqp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_h2f.restype = ctypes.c_float
        _lib.orc_h2f.argtypes = [ctypes.c_uint16]
        _lib.orc_f2h.restype = ctypes.c_uint16
        _lib.orc_f2h.argtypes = [ctypes.c_float]
        _lib.orc_quant_loss.restype = ctypes.c_double
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def h2f(h16):
    h = _c(np.asarray(h16).view(np.uint16).ravel(), np.uint16)
    out = np.empty(h.size, np.float32)
    lib().orc_h2f_array(ctypes.c_size_t(h.size), _p(h), _p(out))
    return out.reshape(np.asarray(h16).shape)


def f2h(f32):
    f = _c(np.asarray(f32, np.float32).ravel(), np.float32)
    out = np.empty(f.size, np.uint16)
    lib().orc_f2h_array(ctypes.c_size_t(f.size), _p(f), _p(out))
    return out.view(np.float16).reshape(np.asarray(f32).shape)


def absmax_x(x):
    x = _c(x, np.float16)
    T, K = x.shape
    ax = np.empty(K, np.float32)
    lib().orc_absmax_x(T, K, _p(x), _p(ax))
    return ax


def absmax_w(w):
    w = _c(w, np.float16)
    K, N = w.shape
    aw = np.empty(K, np.float32)
    lib().orc_absmax_w(K, N, _p(w), _p(aw))
    return aw


def smooth_factor(ax, aw, alpha):
    ax = _c(ax, np.float32)
    aw = _c(aw, np.float32)
    s = np.empty(ax.size, np.float32)
    lib().orc_smooth_factor(ax.size, ctypes.c_float(alpha), _p(ax), _p(aw), _p(s))
    return s


def smooth_scales(xcal, w, alpha):
    xcal = _c(xcal, np.float16)
    w = _c(w, np.float16)
    T, K = xcal.shape
    K2, N = w.shape
    assert K == K2
    s = np.empty(K, np.float32)
    lib().orc_smooth_scales(T, K, N, ctypes.c_float(alpha), _p(xcal), _p(w), _p(s))
    return s


def smooth_apply_x(x, s):
    x = _c(x, np.float16)
    s = _c(s, np.float32)
    M, K = x.shape
    assert s.size == K
    out = np.empty_like(x)
    lib().orc_smooth_apply_x(M, K, _p(x), _p(s), _p(out))
    return out


def smooth_apply_w(w, s):
    w = _c(w, np.float16)
    s = _c(s, np.float32)
    K, N = w.shape
    assert s.size == K
    out = np.empty_like(w)
    lib().orc_smooth_apply_w(K, N, _p(w), _p(s), _p(out))
    return out


def quantize_pack(w, group=128):
    """-> packed uint32 [K/8, N], scales float16 [K/group, N], zeros uint8 [K/group, N]"""
    w = _c(w, np.float16)
    K, N = w.shape
    assert K % group == 0 and group % 8 == 0
    packed = np.empty((K // 8, N), np.uint32)
    scales = np.empty((K // group, N), np.float16)
    zeros = np.empty((K // group, N), np.uint8)
    lib().orc_quantize_pack(N, K, group, _p(w), _p(packed), _p(scales), _p(zeros))
    return packed, scales, zeros


def dequantize(packed, scales, zeros, group=128):
    packed = _c(packed, np.uint32)
    scales = _c(scales, np.float16)
    zeros = _c(zeros, np.uint8)
    K = packed.shape[0] * 8
    N = packed.shape[1]
    out = np.empty((K, N), np.float16)
    lib().orc_dequantize(N, K, group, _p(packed), _p(scales), _p(zeros), _p(out))
    return out


def unpack(packed):
    packed = _c(packed, np.uint32)
    K = packed.shape[0] * 8
    N = packed.shape[1]
    out = np.empty((K, N), np.uint8)
    lib().orc_unpack(N, K, _p(packed), _p(out))
    return out


def w4a16_gemm_ref(x, packed, scales, zeros, group=128):
    """fp64 definition: returns (y [M,N] float64, t [M,N] float64 = sum |x*w_hat|)."""
    x = _c(x, np.float16)
    packed = _c(packed, np.uint32)
    scales = _c(scales, np.float16)
    zeros = _c(zeros, np.uint8)
    M, K = x.shape
    N = packed.shape[1]
    assert packed.shape[0] * 8 == K
    y = np.empty((M, N), np.float64)
    t = np.empty((M, N), np.float64)
    lib().orc_w4a16_gemm_ref(M, N, K, group, _p(x), _p(packed), _p(scales), _p(zeros), _p(y), _p(t))
    return y, t


def w4a16_gemm_f32(x, packed, scales, zeros, group=128):
    """fp32-accumulate, fp16-out variant (the one the CPU baseline times)."""
    x = _c(x, np.float16)
    packed = _c(packed, np.uint32)
    scales = _c(scales, np.float16)
    zeros = _c(zeros, np.uint8)
    M, K = x.shape
    N = packed.shape[1]
    assert packed.shape[0] * 8 == K
    y = np.empty((M, N), np.float16)
    lib().orc_w4a16_gemm_f32(M, N, K, group, _p(x), _p(packed), _p(scales), _p(zeros), _p(y))
    return y


def quant_loss(x, w, x_hat, w_hat):
    x = _c(x, np.float16)
    w = _c(w, np.float16)
    x_hat = _c(x_hat, np.float16)
    w_hat = _c(w_hat, np.float16)
    M, K = x.shape
    N = w.shape[1]
    return float(lib().orc_quant_loss(M, N, K, _p(x), _p(w), _p(x_hat), _p(w_hat)))


def num_threads():
    return int(lib().orc_num_threads())


def ulp16(v):
    """Spacing of fp16 at |v| (subnormal spacing below 2^-14), as float64."""
    a = np.abs(np.asarray(v, np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -14)))
    e = np.clip(e, -14, 15)
    return 2.0 ** (e - 10)


# ---------------------------------------------------------------------------------------------
# LlamaMLP block with the smoothing factors folded into the preceding layers (Sec 2.2, Fig. 5):
# plain fp64 definitions in numpy.  Test infrastructure like the rest of this package.

def rmsnorm_ref(x, gamma, eps):
    """LlamaRMSNorm in fp64: x / sqrt(mean(x^2) + eps) * gamma, rows of x [M,H]; returns float64."""
    x = np.asarray(x, np.float64)
    g = np.asarray(gamma, np.float64)
    r = np.sqrt(np.mean(x * x, axis=1, keepdims=True) + float(eps))
    return x / r * g


def silu_ref(g):
    """SiLU(g) = g * sigmoid(g) = g / (1 + exp(-g)) in fp64."""
    g = np.asarray(g, np.float64)
    return g / (1.0 + np.exp(-g))


def silu_mul_ref(gate, up):
    """The LlamaMLP activation: SiLU(gate) * up, fp64."""
    return silu_ref(gate) * np.asarray(up, np.float64)


def scale_columns(w, s):
    """w[k][n] / s[n]: fp32 divide, one rounding to fp16 (the division of down_proj's input by its
    smoothing factor, folded into up_proj's output columns)."""
    w = _c(w, np.float16)
    s = _c(s, np.float32)
    return (w.astype(np.float32) / s[None, :]).astype(np.float16)


def interleave_gate_up(w_gate, w_up):
    """[K,I] x 2 -> [K,2I] with column 2j = gate j, column 2j+1 = up j (the merged layout whose
    GEMM epilogue can form SiLU(gate) * up from adjacent columns)."""
    w_gate = _c(w_gate, np.float16)
    w_up = _c(w_up, np.float16)
    K, I = w_gate.shape
    out = np.empty((K, 2 * I), np.float16)
    out[:, 0::2] = w_gate
    out[:, 1::2] = w_up
    return out


def mlp_block_ref(x, gamma, eps, w_gate, w_up, w_down):
    """The unquantised, unsmoothed block in fp64: down(SiLU(gate(n)) * up(n)), n = RMSNorm(x)."""
    n = rmsnorm_ref(x, gamma, eps)
    h = silu_mul_ref(n @ np.asarray(w_gate, np.float64), n @ np.asarray(w_up, np.float64))
    return h @ np.asarray(w_down, np.float64)
