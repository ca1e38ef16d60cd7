"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random draws with the shapes and
statistics of the paper's workloads (Code Llama linear layers; flat, small
weights; activation outliers ~100x confined to a few fixed channels, Sec 2.2 and
Figs. 1-2 of arXiv 2312.03788).  The paper's own inputs (Code Llama checkpoints,
HumanEval prompts) are not available; these stand in for them.
"""
import numpy as np

GROUP = 128
ALPHA = 0.5
T_CAL = 512

# (K -> N) of the four merged linears of one decoder layer: qkv, o, gate+up, down
MODEL_SHAPES = {
    "7b": [(4096, 12288), (4096, 4096), (4096, 22016), (11008, 4096)],
    "13b": [(5120, 15360), (5120, 5120), (5120, 27648), (13824, 5120)],
    "34b": [(8192, 10240), (8192, 8192), (8192, 44032), (22016, 8192)],
}
MODEL_LAYERS = {"7b": 32, "13b": 40, "34b": 48}
MODEL_DECODE_M = {"7b": [1, 8, 16], "13b": [1, 16, 64], "34b": [1, 16, 64, 256]}
PREFILL_M = [2048, 4096]


def outlier_channels(K, frac=0.01, seed=7):
    """Fixed set of outlier input channels (the same for every token)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = int(round(frac * K))
    return np.sort(rng.choice(K, size=n, replace=False))


def weight(K, N, seed, sigma=0.02):
    """W[K, N] fp16 ~ N(0, sigma)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(sigma)
    return w.astype(np.float16)


def activation(M, K, seed, outlier_gain=50.0):
    """X[M, K] fp16 ~ N(0, 1), the outlier channels scaled by `outlier_gain`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((M, K), dtype=np.float32)
    x[:, outlier_channels(K)] *= np.float32(outlier_gain)
    return x.astype(np.float16)


def layer_inputs(M, K, N, layer=0, shape_idx=0):
    """(X[M,K], Xcal[T_CAL,K], W[K,N]) for one linear layer, all fp16."""
    w = weight(K, N, seed=1000 + 16 * layer + shape_idx)
    x = activation(M, K, seed=2000 + M)
    xcal = activation(T_CAL, K, seed=3000)
    return x, xcal, w


def algorithmic_bytes(M, N, K, group=GROUP):
    """Bytes the method itself must move for one W4A16 GEMM: 4-bit codes, one
    fp16 step and one 4-bit zero point per group, fp16 X in and fp16 Y out."""
    return N * K * (0.5 + 2.0 / group + 0.5 / group) + 2.0 * M * K + 2.0 * M * N


def gemm_flops(M, N, K):
    return 2.0 * M * N * K
