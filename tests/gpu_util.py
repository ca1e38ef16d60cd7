"""Helpers for the GPU parity tests: move numpy arrays to the device, run the HIP path
through the C ABI binding, bring results back as numpy."""
import numpy as np
import torch


def dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    a = t.detach().cpu().numpy()
    return a


def host_u32(t):
    return host(t).view(np.uint32)


def gemm_tolerance_ok(orc, y_gpu, y_ref, t_ref):
    """|y_gpu - y_ref| <= 1e-3 * sum_k |x w_hat| + 1 fp16 ulp, per element."""
    err = np.abs(y_gpu.astype(np.float64) - y_ref)
    tol = 1e-3 * t_ref + orc.ulp16(y_ref)
    bad = err > tol
    return not bad.any(), float((err / tol).max()), int(bad.sum())
