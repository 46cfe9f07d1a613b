"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds NO arithmetic of the method: it only draws random activations
and random sparse Winograd-domain weights and lays the latter out as per-position
CSR.  Both the GPU library and the CPU oracle are fed the arrays it returns.

The shapes, densities and value distributions stand in for the workloads of the
paper's Section 6.2 (3x3 and 5x5 layers of an AlexNet pruned natively in the Winograd
domain, Table 1 method A: 4-10 % non-zeros), whose trained weights and dataset
are not available: post-ReLU-like activations ``max(0, N(0,1))``, iid Bernoulli
masks, non-zeros ``N(0, sigma=0.05)``.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 170208597

# name -> layer shape + weight recipe.  "bench" is the configuration the metric is quoted on.
CONFIGS = {
    "alexnet_conv3_n1_f2": dict(N=1, C=256, H=13, W=13, K=384, m=2, r=3, pad=1, density=0.10, seed=BASE_SEED + 0),
    "alexnet_conv3_n32_f4": dict(N=32, C=256, H=13, W=13, K=384, m=4, r=3, pad=1, density=0.10, seed=BASE_SEED + 1),
    "alexnet_conv3_n64_f4": dict(N=64, C=256, H=13, W=13, K=384, m=4, r=3, pad=1, density=0.10, seed=BASE_SEED + 2),
    "alexnet_conv4_n64_f4": dict(N=64, C=384, H=13, W=13, K=384, m=4, r=3, pad=1, density=0.10, seed=BASE_SEED + 3),
    "alexnet_conv5_n64_f4": dict(N=64, C=384, H=13, W=13, K=256, m=4, r=3, pad=1, density=0.10, seed=BASE_SEED + 4),
    "vgg_56_n32_f4": dict(N=32, C=256, H=56, W=56, K=256, m=4, r=3, pad=1, density=0.10, seed=BASE_SEED + 5),
    # one of the two channel groups of AlexNet's 5x5 layer (Table 1: conv2, 90.6 % sparse under method A)
    "alexnet_conv2g_n32_f2r5": dict(N=32, C=48, H=27, W=27, K=128, m=2, r=5, pad=2, density=0.094, seed=BASE_SEED + 7),
    "alexnet_conv2g_n32_f4r5": dict(N=32, C=48, H=27, W=27, K=128, m=4, r=5, pad=2, density=0.094, seed=BASE_SEED + 8),
    "conv4_skewed_n64_f4": dict(N=64, C=384, H=13, W=13, K=384, m=4, r=3, pad=1, density=None, seed=BASE_SEED + 6),
}
BENCH_CONFIG = "vgg_56_n32_f4"
DENSITY_SWEEP = (0.30, 0.20, 0.10, 0.05)


def geometry(N, C, H, W, K, m, r, pad):
    """Derived sizes: t, P, Ho, Wo, th, tw, T (pure index bookkeeping)."""
    t = m + r - 1
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    th, tw = -(-Ho // m), -(-Wo // m)
    return dict(t=t, P=t * t, Ho=Ho, Wo=Wo, th=th, tw=tw, T=N * th * tw)


def direct_conv_flops(N, C, H, W, K, m, r, pad):
    """FLOPs a dense direct convolution would execute (the paper's effective-FLOP numerator)."""
    g = geometry(N, C, H, W, K, m, r, pad)
    return 2 * N * K * C * g["Ho"] * g["Wo"] * r * r


def activations(N, C, H, W, seed):
    """Post-ReLU-like feature maps: max(0, z), z ~ N(0,1), fp32 NCHW."""
    rng = np.random.default_rng(seed)
    return np.maximum(rng.standard_normal((N, C, H, W), dtype=np.float32), np.float32(0))


def dense_to_csr(mask, values):
    """mask, values: [P][K][C] -> (rowptr[P*K+1], colidx, vals); rows are p*K+k, columns ascending."""
    P, K, C = mask.shape
    m2 = mask.reshape(P * K, C)
    counts = m2.sum(axis=1, dtype=np.int64)
    rowptr = np.zeros(P * K + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    _, cols = np.nonzero(m2)
    vals = values.reshape(P * K, C)[m2]
    return rowptr.astype(np.int32), cols.astype(np.int32), np.ascontiguousarray(vals)


def bernoulli_weights(P, K, C, density, seed, sigma=0.05):
    """iid Bernoulli(density) mask over [P][K][C], non-zeros ~ N(0, sigma), as per-position CSR."""
    rng = np.random.default_rng(seed)
    mask = rng.random((P, K, C), dtype=np.float32) < np.float32(density)
    values = (rng.standard_normal((P, K, C), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    return dense_to_csr(mask, values)


def skewed_weights(P, K, C, seed, sigma=0.05, lo=0.01, hi=0.30, zipf=1.2):
    """Load-imbalance stress: per-position density ~ U[lo,hi]; per-row density follows a
    Zipf(zipf) profile over a random ranking of the K rows, clipped at 1 and rescaled so the
    position's mean row density equals its drawn density."""
    rng = np.random.default_rng(seed)
    d_p = rng.uniform(lo, hi, size=P)
    mask = np.zeros((P, K, C), dtype=bool)
    for p in range(P):
        rank = rng.permutation(K) + 1
        raw = rank.astype(np.float64) ** (-zipf)
        scale = d_p[p] * K / raw.sum()
        for _ in range(200):
            rho = np.minimum(1.0, scale * raw)
            scale *= d_p[p] / rho.mean()
        rho = np.minimum(1.0, scale * raw)
        mask[p] = rng.random((K, C)) < rho[:, None]
    values = (rng.standard_normal((P, K, C), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    return dense_to_csr(mask, values)


def dense_weights(P, K, C, seed, sigma=0.05):
    """0 %-sparsity comparison weights, [P][K][C] ~ N(0, sigma)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((P, K, C), dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def integer_case(N, C, H, W, K, m, r, density, seed):
    """Small-integer data (inputs in {0..3}, weights in {-2..2}, stored zeros included): every
    intermediate is an integer far below 2**24, so fp32 results are exact in any summation order."""
    rng = np.random.default_rng(seed)
    t = m + r - 1
    P = t * t
    x = rng.integers(0, 4, size=(N, C, H, W)).astype(np.float32)
    mask = rng.random((P, K, C)) < density
    values = rng.integers(-2, 3, size=(P, K, C)).astype(np.float32)
    return (x,) + dense_to_csr(mask, values)


def make_layer(name, density=None, N=None):
    """Build (cfg, in, rowptr, colidx, vals) for a named configuration."""
    cfg = dict(CONFIGS[name])
    if density is not None:
        cfg["density"] = density
    if N is not None:
        cfg["N"] = N
    g = geometry(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
    x = activations(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["seed"])
    if cfg["density"] is None:
        rp, ci, va = skewed_weights(g["P"], cfg["K"], cfg["C"], cfg["seed"] + 1000)
    else:
        rp, ci, va = bernoulli_weights(g["P"], cfg["K"], cfg["C"], cfg["density"], cfg["seed"] + 1000)
    cfg.update(g)
    return cfg, x, rp, ci, va
