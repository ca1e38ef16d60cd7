"""ctypes binding of libsqp.so (see include/sqp.h for the contract of each call).

Same names as the C entry points without the ``sqp_`` prefix.  Tensors must live on
the GPU, be contiguous and have the dtype the C ABI expects; outputs are allocated
with torch (device memory plumbing only) unless passed in.
"""
import ctypes
import os

import torch  # also makes sure the process-wide HIP runtime is the one torch uses

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("SQP_LIBRARY", os.path.join(_HERE, "libsqp.so"))  # override: another build

EXPORTS = ["sqp_status_string", "sqp_smooth_scales", "sqp_smooth_apply_x", "sqp_smooth_apply_w",
           "sqp_quantize_pack", "sqp_dequantize", "sqp_w4a16_gemm", "sqp_quant_loss", "sqp_transpose_nk",
           "sqp_w4a16_gemm_silu_mul", "sqp_rmsnorm", "sqp_scale_columns", "sqp_interleave_gate_up",
           "sqp_set_workspace", "sqp_alpha_search", "sqp_w4a16_gemm_static"]


class SqpError(RuntimeError):
    pass


_lib = None


def lib():
    """Load libsqp.so (built beforehand by paper_2312_03788_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise SqpError("libsqp.so is not built: run `python -m paper_2312_03788_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.sqp_status_string.restype = ctypes.c_char_p
        L.sqp_status_string.argtypes = [ctypes.c_int]
        vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.sqp_smooth_scales.argtypes = [i, i, i, f, vp, vp, vp, vp]
        L.sqp_smooth_apply_x.argtypes = [i, i, vp, vp, vp, vp]
        L.sqp_smooth_apply_w.argtypes = [i, i, vp, vp, vp, vp]
        L.sqp_quantize_pack.argtypes = [i, i, i, vp, vp, vp, vp, vp]
        L.sqp_dequantize.argtypes = [i, i, i, vp, vp, vp, vp, vp]
        L.sqp_w4a16_gemm.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp]
        L.sqp_quant_loss.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.sqp_transpose_nk.argtypes = [i, i, vp, vp, vp]
        L.sqp_w4a16_gemm_silu_mul.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp]
        L.sqp_w4a16_gemm_static.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp]
        L.sqp_rmsnorm.argtypes = [i, i, vp, vp, f, vp, vp]
        L.sqp_scale_columns.argtypes = [i, i, vp, vp, vp, vp]
        L.sqp_interleave_gate_up.argtypes = [i, i, vp, vp, vp, vp]
        L.sqp_quant_loss_scratch_doubles.argtypes = [i, i]
        L.sqp_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
        L.sqp_alpha_search.argtypes = [i, i, i, i, i, ctypes.POINTER(ctypes.c_float)] + [vp] * 13
        L.sqp_w4a16_gemm_workspace_bytes.argtypes = [i, i, i, i]
        L.sqp_w4a16_gemm_workspace_bytes.restype = ctypes.c_size_t
        for name in EXPORTS[1:]:
            getattr(L, name).restype = ctypes.c_int
        L.sqp_quant_loss_scratch_doubles.restype = ctypes.c_long
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise SqpError("%s failed: %s (%d)" % (what, lib().sqp_status_string(rc).decode(), rc))


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda):
        raise SqpError("%s must be a GPU tensor" % name)
    if t.dtype != dtype:
        raise SqpError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise SqpError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_workspaces = {}  # device index -> torch buffer handed to the library (kept alive here)


def set_workspace(nbytes, device=None):
    """Allocate a device buffer of `nbytes` with torch and hand it to the library as the
    workspace for split launches of the GEMM on that device (sqp_set_workspace).  0 removes it.
    Buffers set earlier stay referenced until the process ends: launches already enqueued
    may still use them."""
    dev = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    with torch.cuda.device(dev):
        if nbytes <= 0:
            _check(lib().sqp_set_workspace(None, 0, _stream()), "sqp_set_workspace")
            _workspaces.setdefault(dev.index, []).append(None)
            return None
        buf = torch.empty(int(nbytes), dtype=torch.uint8, device=dev)
        _check(lib().sqp_set_workspace(ctypes.c_void_p(buf.data_ptr()), int(nbytes), _stream()), "sqp_set_workspace")
        _workspaces.setdefault(dev.index, []).append(buf)
    return buf


def workspace_bytes(M, N, K, group=128):
    """Bytes of workspace the launch plan of the GEMM uses for this shape (0: none)."""
    return int(lib().sqp_w4a16_gemm_workspace_bytes(M, N, K, group))


def _ensure_workspace(M, N, K, group, device):
    """Device-memory plumbing for the GEMM calls: make sure the workspace set on the tensor's
    device covers this shape's plan (grown with some slack so that a sweep over shapes
    settles after a few calls).  Callers that must not allocate (graph capture) call
    set_workspace themselves beforehand."""
    need = workspace_bytes(M, N, K, group)
    if need == 0:
        return
    held = _workspaces.get(device.index)
    have = held[-1].numel() if held and held[-1] is not None else 0
    if need > have:
        set_workspace(max(need, 2 * have, 16 << 20), device)


def smooth_scales(x_cal, w, alpha, out=None):
    """Eq. 6: s [K] fp32 from calibration activations x_cal [T,K] and weight w [K,N]."""
    T, K = x_cal.shape
    K2, N = w.shape
    if K != K2:
        raise SqpError("x_cal and w disagree on K")
    s = out if out is not None else torch.empty(K, dtype=torch.float32, device=w.device)
    _check(lib().sqp_smooth_scales(T, K, N, float(alpha), _dev(x_cal, torch.float16, "x_cal"),
                                   _dev(w, torch.float16, "w"), _dev(s, torch.float32, "s"), _stream()),
           "sqp_smooth_scales")
    return s


def smooth_apply_x(x, s, out=None):
    """Eq. 5, activation side: x / s per input channel."""
    M, K = x.shape
    o = out if out is not None else torch.empty_like(x)
    _check(lib().sqp_smooth_apply_x(M, K, _dev(x, torch.float16, "x"), _dev(s, torch.float32, "s"),
                                    _dev(o, torch.float16, "x_out"), _stream()), "sqp_smooth_apply_x")
    return o


def smooth_apply_w(w, s, out=None):
    """Eq. 5, weight side: s * w per input channel."""
    K, N = w.shape
    o = out if out is not None else torch.empty_like(w)
    _check(lib().sqp_smooth_apply_w(K, N, _dev(w, torch.float16, "w"), _dev(s, torch.float32, "s"),
                                    _dev(o, torch.float16, "w_out"), _stream()), "sqp_smooth_apply_w")
    return o


def quantize_pack(w, group=128, out=None):
    """Eq. 1 group-wise along K: returns (packed int32 [K/8,N] holding the uint32 words,
    scales fp16 [K/group,N], zeros uint8 [K/group,N])."""
    K, N = w.shape
    if out is not None:
        packed, scales, zeros = out
    else:
        if group <= 0 or K % max(group, 1):
            raise SqpError("K must be a multiple of group")
        packed = torch.empty((K // 8, N), dtype=torch.int32, device=w.device)
        scales = torch.empty((K // group, N), dtype=torch.float16, device=w.device)
        zeros = torch.empty((K // group, N), dtype=torch.uint8, device=w.device)
    _check(lib().sqp_quantize_pack(N, K, group, _dev(w, torch.float16, "w"), _dev(packed, torch.int32, "packed"),
                                   _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                                   _stream()), "sqp_quantize_pack")
    return packed, scales, zeros


def dequantize(packed, scales, zeros, group=128, out=None):
    """Second line of Eq. 1: w_hat fp16 [K,N]."""
    K, N = packed.shape[0] * 8, packed.shape[1]
    o = out if out is not None else torch.empty((K, N), dtype=torch.float16, device=packed.device)
    _check(lib().sqp_dequantize(N, K, group, _dev(packed, torch.int32, "packed"), _dev(scales, torch.float16, "scales"),
                                _dev(zeros, torch.uint8, "zeros"), _dev(o, torch.float16, "w_hat"), _stream()),
           "sqp_dequantize")
    return o


def w4a16_gemm(x, packed, scales, zeros, group=128, out=None):
    """Eq. 3: y [M,N] fp16 = x [M,K] fp16 times the group-wise 4-bit weight."""
    M, K = x.shape
    N = packed.shape[1]
    if packed.shape[0] * 8 != K:
        raise SqpError("x and packed disagree on K")
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    _ensure_workspace(M, N, K, group, x.device)
    _check(lib().sqp_w4a16_gemm(M, N, K, group, _dev(x, torch.float16, "x"), _dev(packed, torch.int32, "packed"),
                                _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                                _dev(y, torch.float16, "y"), _stream()), "sqp_w4a16_gemm")
    return y


def w4a16_gemm_static(x, packed, scales, zeros, group=128, out=None):
    """Eq. 3 through the entry point that allocates nothing and needs no workspace (partial
    sums in the library's static device array); `out` should be passed by callers that must
    not allocate."""
    M, K = x.shape
    N = packed.shape[1]
    if packed.shape[0] * 8 != K:
        raise SqpError("x and packed disagree on K")
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().sqp_w4a16_gemm_static(M, N, K, group, _dev(x, torch.float16, "x"), _dev(packed, torch.int32, "packed"),
                                       _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                                       _dev(y, torch.float16, "y"), _stream()), "sqp_w4a16_gemm_static")
    return y


def w4a16_gemm_silu_mul(x, packed, scales, zeros, group=128, out=None):
    """Merged, interleaved gate/up projection with SiLU(gate) * up fused: y [M, N/2] fp16."""
    M, K = x.shape
    N = packed.shape[1]
    if packed.shape[0] * 8 != K:
        raise SqpError("x and packed disagree on K")
    y = out if out is not None else torch.empty((M, N // 2), dtype=torch.float16, device=x.device)
    _ensure_workspace(M, N, K, group, x.device)
    _check(lib().sqp_w4a16_gemm_silu_mul(M, N, K, group, _dev(x, torch.float16, "x"), _dev(packed, torch.int32, "packed"),
                                         _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                                         _dev(y, torch.float16, "y"), _stream()), "sqp_w4a16_gemm_silu_mul")
    return y


def rmsnorm(x, gamma, eps, out=None):
    """LlamaRMSNorm with an fp16 weight (possibly already divided by a smoothing factor)."""
    M, H = x.shape
    y = out if out is not None else torch.empty_like(x)
    _check(lib().sqp_rmsnorm(M, H, _dev(x, torch.float16, "x"), _dev(gamma, torch.float16, "gamma"), float(eps),
                             _dev(y, torch.float16, "y"), _stream()), "sqp_rmsnorm")
    return y


def scale_columns(w, s, out=None):
    """w[k][n] / s[n] in fp16: a smoothing factor folded into the producing layer's columns."""
    K, N = w.shape
    o = out if out is not None else torch.empty_like(w)
    _check(lib().sqp_scale_columns(K, N, _dev(w, torch.float16, "w"), _dev(s, torch.float32, "s"),
                                   _dev(o, torch.float16, "w_out"), _stream()), "sqp_scale_columns")
    return o


def interleave_gate_up(w_gate, w_up, out=None):
    """[K,I] x 2 -> [K,2I], column 2j = gate j, column 2j+1 = up j."""
    K, I = w_gate.shape
    o = out if out is not None else torch.empty((K, 2 * I), dtype=torch.float16, device=w_gate.device)
    _check(lib().sqp_interleave_gate_up(K, I, _dev(w_gate, torch.float16, "w_gate"), _dev(w_up, torch.float16, "w_up"),
                                        _dev(o, torch.float16, "w_out"), _stream()), "sqp_interleave_gate_up")
    return o


def transpose_nk(w_nk, out=None):
    """[N,K] fp16 (checkpoint orientation) -> [K,N] fp16 (the orientation of Eq. 2)."""
    N, K = w_nk.shape
    o = out if out is not None else torch.empty((K, N), dtype=torch.float16, device=w_nk.device)
    _check(lib().sqp_transpose_nk(N, K, _dev(w_nk, torch.float16, "w_nk"), _dev(o, torch.float16, "w_kn"), _stream()),
           "sqp_transpose_nk")
    return o


def quant_loss(x, w, x_hat, packed, scales, zeros, group=128, out=None):
    """Eq. 4 for one layer: ||x w - x_hat w_hat||_F^2 as a one-element fp64 GPU tensor."""
    M, K = x.shape
    N = w.shape[1]
    if w.shape[0] != K or tuple(x_hat.shape) != (M, K) or packed.shape[0] * 8 != K or packed.shape[1] != N:
        raise SqpError("x, w, x_hat and packed disagree on the shape")
    L = lib()
    scratch = torch.empty(int(L.sqp_quant_loss_scratch_doubles(M, N)), dtype=torch.float64, device=x.device)
    o = out if out is not None else torch.empty(1, dtype=torch.float64, device=x.device)
    _check(L.sqp_quant_loss(M, N, K, group, _dev(x, torch.float16, "x"), _dev(w, torch.float16, "w"),
                            _dev(x_hat, torch.float16, "x_hat"), _dev(packed, torch.int32, "packed"),
                            _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                            _dev(scratch, torch.float64, "scratch"), _dev(o, torch.float64, "loss"), _stream()),
           "sqp_quant_loss")
    return o


def alpha_search(x_cal, w, group=128, alphas=None):
    """Single-layer search for the smoothing strength (Sec 2.2) through sqp_alpha_search: the
    per-channel maxima once, then Eq. 6 -> Eq. 5 -> Eq. 1 -> Eq. 4 per alpha and the argmin, all
    in library kernels.  Returns (best alpha, list of (alpha, loss))."""
    if alphas is None:
        alphas = [0.05 * i for i in range(21)]
    T, K = x_cal.shape
    N = w.shape[1]
    if w.shape[0] != K or group <= 0 or K % group:
        raise SqpError("x_cal, w and group disagree on K")
    L = lib()
    dev = w.device
    n = len(alphas)
    host_alphas = (ctypes.c_float * n)(*[float(a) for a in alphas])
    amax = torch.empty(2 * K, dtype=torch.float32, device=dev)
    s = torch.empty(K, dtype=torch.float32, device=dev)
    xh = torch.empty_like(x_cal)
    ws = torch.empty_like(w)
    packed = torch.empty((K // 8, N), dtype=torch.int32, device=dev)
    scales = torch.empty((K // group, N), dtype=torch.float16, device=dev)
    zeros = torch.empty((K // group, N), dtype=torch.uint8, device=dev)
    scratch = torch.empty(int(L.sqp_quant_loss_scratch_doubles(T, N)), dtype=torch.float64, device=dev)
    loss = torch.empty(n, dtype=torch.float64, device=dev)
    best = torch.empty(1, dtype=torch.int32, device=dev)
    _check(L.sqp_alpha_search(T, N, K, group, n, host_alphas, _dev(x_cal, torch.float16, "x_cal"), _dev(w, torch.float16, "w"),
                              _dev(amax, torch.float32, "amax"), _dev(s, torch.float32, "s"), _dev(xh, torch.float16, "x_hat"),
                              _dev(ws, torch.float16, "w_s"), _dev(packed, torch.int32, "packed"),
                              _dev(scales, torch.float16, "scales"), _dev(zeros, torch.uint8, "zeros"),
                              _dev(scratch, torch.float64, "scratch"), _dev(loss, torch.float64, "loss"),
                              _dev(best, torch.int32, "best"), _stream()), "sqp_alpha_search")
    vals = [float(v) for v in loss.cpu()]
    b = int(best.cpu()[0])
    return float(alphas[b]), list(zip([float(a) for a in alphas], vals))
