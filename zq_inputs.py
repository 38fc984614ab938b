"""Seeded synthetic inputs for the quantized-linear workloads.

This module only draws random tensors; it holds none of the method's
arithmetic (no quantizer, no normalisation, no matmul) and imports neither the
GPU library nor the oracle.  Both sides are fed from here.

The paper evaluates on trained BERT / GPT checkpoints and real text; none of
that is available, so the tensors below stand in for it.  They reproduce the
structure the paper reports for those models:
  * activations with a few large-magnitude channels and a spread of per-token
    ranges (Sec. 3, Fig. 1: token ranges differ several-fold),
  * weight rows whose magnitudes differ by about 10x (Sec. 3),
  * the layer shapes and group counts of App. B.2 (48 groups BERT-base, 64
    BERT-large, 64/128 for GPT-3 350M/1.3B).
All values are rounded to fp16, which is what the layer receives.
"""
import numpy as np

BASE_SEED = 220601861


def rng_for(config, index=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 100 * config + index))


# name -> (K, N, groups, weight bits)
LINEARS = {
    "c1": (768, 768, 48, 8),
    "c2_ffc1": (1024, 4096, 64, 8),
    "c2_ffc2": (4096, 1024, 64, 8),
    "c3_qkv": (2048, 6144, 128, 8),
    "c3_out": (2048, 2048, 128, 8),
    "c3_ffc1": (2048, 8192, 128, 8),
    "c3_ffc2": (8192, 2048, 128, 8),
    "c4_ffc1": (4096, 16384, 256, 4),
    "c4_ffc2": (16384, 4096, 256, 4),
    "c4_qkv": (4096, 12288, 256, 8),
    "c4_out": (4096, 4096, 256, 8),
    "c5_qkv": (6144, 18432, 192, 8),
    "c5_ffc1": (6144, 24576, 192, 8),
    "c5_ffc2": (24576, 6144, 192, 8),
    "c5_out": (6144, 6144, 192, 8),       # the attention output projection of the same layer (the configuration lists none)
}

# token counts each configuration is exercised at
TOKENS = {
    "c1": (128,),
    "c2": (4096,),
    "c3": (1, 8, 32, 2048),
    "c4": (1, 16, 4096),
    "c5": (64, 16384),
}


def weights(rng, N, K, row_spread=True, std=0.02):
    """fp16 [N,K] ~ N(0, std^2), rows scaled by a log-uniform factor in [0.3, 3]."""
    w = rng.standard_normal((N, K), dtype=np.float32) * np.float32(std)
    if row_spread:
        f = np.exp(rng.uniform(np.log(0.3), np.log(3.0), size=(N, 1))).astype(np.float32)
        w *= f
    return w.astype(np.float16)


def bias(rng, N, std=0.01):
    return (rng.standard_normal(N, dtype=np.float32) * np.float32(std)).astype(np.float16)


def layernorm_params(rng, K):
    g = (1.0 + 0.1 * rng.standard_normal(K, dtype=np.float32)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K, dtype=np.float32)).astype(np.float16)
    return g, b


def activations(rng, M, K, outlier_frac=0.0, outlier_scale=1.0, n_outliers=None,
                token_spread=False, heavy_tail_frac=0.0):
    """fp16 [M,K] ~ N(0,1) with structured outliers.

    outlier channels: n_outliers (or outlier_frac*K) fixed columns times outlier_scale
    token_spread:     per-token std log-uniform in [0.5, 2]
    heavy_tail_frac:  that fraction of columns replaced by Student-t(df=3) draws
    """
    x = rng.standard_normal((M, K), dtype=np.float32)
    if token_spread:
        f = np.exp(rng.uniform(np.log(0.5), np.log(2.0), size=(M, 1))).astype(np.float32)
        x *= f
    n_out = n_outliers if n_outliers is not None else int(round(outlier_frac * K))
    if n_out > 0:
        cols = rng.choice(K, size=n_out, replace=False)
        x[:, cols] *= np.float32(outlier_scale)
    n_ht = int(round(heavy_tail_frac * K))
    if n_ht > 0:
        cols = rng.choice(K, size=n_ht, replace=False)
        x[:, cols] = rng.standard_t(3.0, size=(M, n_ht)).astype(np.float32)
    return x.astype(np.float16)


def config_activations(cfg, rng, M, K):
    """Activation recipe of configuration cfg ('c1'..'c5')."""
    if cfg == "c1":
        return activations(rng, M, K, n_outliers=4, outlier_scale=20.0)
    if cfg == "c2":
        return activations(rng, M, K, outlier_frac=0.01, outlier_scale=15.0)
    if cfg == "c3" or cfg == "c5":
        return activations(rng, M, K, token_spread=True)
    if cfg == "c4":
        return activations(rng, M, K, heavy_tail_frac=0.005)
    raise KeyError(cfg)


def random_codes(rng, shape, qmax=127):
    """Uniform integer codes in [-qmax, qmax]: inputs for GeMM-only cases."""
    return rng.integers(-qmax, qmax + 1, size=shape, dtype=np.int8)


def random_scales(rng, n, lo=1e-3, hi=1e-1):
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n)).astype(np.float32)
