"""Seeded synthetic inputs shaped like the paper's workloads.

Holds no RaZeR arithmetic: only random tensors and the bf16 <-> fp32 bit
conversions needed to hand identical inputs to the CPU oracle and to the HIP
library.  The paper's kernels are measured on the linear projections of
Llama / Qwen models (App. D.2); no model weights exist here, so heavy-tailed
random matrices of the same shapes stand in for them.
"""
import numpy as np

# (name, N = out features, K = in features); W is stored [N][K].
LLAMA_7B_LAYER = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                  ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA_70B_LAYER = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                   ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def weight(n, k, seed, outlier_frac=0.0, outlier_gain=20.0, chunk_rows=2048):
    """fp32 [n][k]: Student-t(nu=4) scaled to std 0.02; a fraction of the
    columns (input channels) multiplied by outlier_gain."""
    rng = np.random.default_rng(seed)
    w = np.empty((n, k), np.float32)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        w[r0:r1] = (rng.standard_t(4.0, size=(r1 - r0, k)) * (0.02 / np.sqrt(2.0))).astype(np.float32)
    n_out = int(round(outlier_frac * k))
    if n_out:
        cols = np.random.default_rng(seed + 7919).choice(k, size=n_out, replace=False)
        w[:, cols] *= np.float32(outlier_gain)
    return w


def activation(m, k, seed, outlier_frac=0.0, outlier_gain=50.0):
    """bf16 bits [m][k]: N(0,1); a fraction of channels multiplied by outlier_gain."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=(m, k)).astype(np.float32)
    n_out = int(round(outlier_frac * k))
    if n_out:
        cols = np.random.default_rng(seed + 7919).choice(k, size=n_out, replace=False)
        a[:, cols] *= np.float32(outlier_gain)
    return f32_to_bf16_bits(a)


def sample_indices(total, count, seed):
    """Sorted distinct indices for sampled checks of large outputs."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(total, size=min(count, total), replace=False)).astype(np.int64)
