"""Seeded synthetic inputs with the shapes and structure of the paper's workloads.

The paper quantizes key / value projection outputs of LLMs on SlimPajama text
(Section 3); neither the models nor the data are available, so these
generators stand in for them.  They keep what the paper reports about the
data: one row per token, d channels per row, and key activations with a few
outlier channels (the reason Section 3.1 gives for grouping channels that are
d/dhat apart).

This module holds NO arithmetic of the method (no std scaling, grouping,
distance, codeword or moving-average code): it only draws numbers and converts
storage types.  It is the one module that both the CPU oracle's tests and the
GPU library's tests/benchmarks may import.

Every generator is driven by ``numpy.random.Generator(PCG64(seed))`` with
``seed = BASE_SEED + workload index`` and sub-streams taken with ``spawn`` in
the order the fields are documented.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 241015704


def _rng(index: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + index + 1000 * extra))


# ----------------------------------------------------------------------------- storage helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored array ('fp32' | 'bf16' (uint16 bits) | 'fp16') to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    if dtype in ("fp32", "fp16"):
        return np.asarray(a).astype(np.float64)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- workload 1
def tiny_kv(N: int = 4096, d: int = 128, n_outlier: int = 4, outlier_scale: float = 10.0,
            index: int = 1):
    """Workload 1: X[N][d] float32 ~ N(0,1), n_outlier seeded channels scaled by outlier_scale.
    Sub-streams: (values, outlier channel permutation).  Returns (X, outlier_channels)."""
    s_val, s_perm = _rng(index).spawn(2)
    X = s_val.standard_normal((N, d), dtype=np.float32)
    ch = np.sort(s_perm.permutation(d)[:n_outlier])
    X[:, ch] *= np.float32(outlier_scale)
    return X, ch


# ----------------------------------------------------------------------------- workload 2
def llama_key(N: int = 32768, d: int = 1024, n_outlier: int = 20, outlier_scale: float = 20.0,
              index: int = 2, rows: slice | None = None):
    """Workload 2 (Llama-3-8B-like key projection, 8 KV heads x 128): bf16( g * sigma_c * o_c ),
    g ~ N(0,1), sigma_c = exp(N(0,1)) per channel, o_c = outlier_scale on exactly n_outlier
    seeded channels (about 2 %), else 1.  Sub-streams: (channel sigma, outlier permutation,
    values).  Returns (bits uint16 [N][d], sigma_c * o_c float32 [d]).
    `rows` limits generation to a prefix slice(0, n) of the rows (same values as the full draw
    for those rows, because values are drawn row-major from one stream)."""
    s_sig, s_perm, s_val = _rng(index).spawn(3)
    sigma = np.exp(s_sig.standard_normal(d)).astype(np.float32)
    ch = np.sort(s_perm.permutation(d)[:n_outlier])
    sigma[ch] *= np.float32(outlier_scale)
    n = N if rows is None else rows.stop
    g = s_val.standard_normal((n, d), dtype=np.float32)
    g *= sigma[None, :]
    return f32_to_bf16_bits(g), sigma


# ----------------------------------------------------------------------------- workload 3
def decode_codebooks(n_sets: int, depth: int = 8, K: int = 2048, dhat: int = 32,
                     shrink: float = 0.6, index: int = 3):
    """Workload 3 codebooks: n_sets independent sets, stage i entries ~ N(0, shrink^(2 i)),
    float32 [n_sets][depth][K][dhat]."""
    rng = _rng(index)
    C = rng.standard_normal((n_sets, depth, K, dhat), dtype=np.float32)
    C *= (np.float32(shrink) ** np.arange(depth, dtype=np.float32))[None, :, None, None]
    return C


def decode_std_fp16(T: int, index: int = 3, extra: int = 1):
    """Workload 3 per-token std, fp16( exp(0.5 * N(0,1)) ), [T]."""
    rng = _rng(index, extra)
    return np.exp(0.5 * rng.standard_normal(T, dtype=np.float32)).astype(np.float16)


def uniform_codes_host(T: int, G: int = 32, depth: int = 8, K: int = 2048, index: int = 3,
                       extra: int = 2):
    """Uniform codes in [0, K), int16 [T][G][depth], drawn on the host."""
    rng = _rng(index, extra)
    return rng.integers(0, K, size=(T, G, depth), dtype=np.int16)


def uniform_codes_device(T: int, G: int, depth: int, K: int, device, index: int = 3,
                         extra: int = 0):
    """Uniform codes in [0, K), int16 [T][G][depth], drawn by torch's seeded generator on
    `device` (the full decode workload is 16 GiB of codes: too large to ship from the host)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(BASE_SEED + index + 1000 * extra)
    return torch.randint(0, K, (T, G, depth), dtype=torch.int16, device=device, generator=gen)


# ----------------------------------------------------------------------------- workload 4
def gaussian_mixture(M: int = 1048576, dhat: int = 32, n_comp: int = 64, sigma: float = 0.3,
                     index: int = 4):
    """Workload 4: R[M][dhat] float32 from n_comp isotropic Gaussians (means ~ N(0,1), std sigma,
    weights ~ Dirichlet(1)).  Sub-streams: (means, weights, component draw, noise)."""
    s_mu, s_w, s_comp, s_noise = _rng(index).spawn(4)
    mu = s_mu.standard_normal((n_comp, dhat)).astype(np.float32)
    w = s_w.dirichlet(np.ones(n_comp))
    comp = s_comp.choice(n_comp, size=M, p=w)
    R = s_noise.standard_normal((M, dhat), dtype=np.float32)
    R *= np.float32(sigma)
    R += mu[comp]
    return R


# ----------------------------------------------------------------------------- workload 5
def heavy_tailed_keys(N: int = 131072, d: int = 4096, alpha: float = 1.5, cap: float = 100.0,
                      index: int = 5, rows: slice | None = None):
    """Workload 5 (long-context MHA, 32 heads x 128): fp16( N(0,1) * sigma_c ),
    sigma_c = min(cap, (1-U)^(-1/alpha)) (Pareto, heavy tailed).
    Sub-streams: (channel sigma, values).  Returns (X float16 [N][d], sigma float32 [d])."""
    s_sig, s_val = _rng(index).spawn(2)
    u = s_sig.random(d)
    sigma = np.minimum(cap, (1.0 - u) ** (-1.0 / alpha)).astype(np.float32)
    n = N if rows is None else rows.stop
    out = np.empty((n, d), dtype=np.float16)
    step = 8192
    for a in range(0, n, step):
        b = min(n, a + step)
        g = s_val.standard_normal((b - a, d), dtype=np.float32)
        g *= sigma[None, :]
        out[a:b] = g.astype(np.float16)
    return out, sigma


# ----------------------------------------------------------------------------- small generic cases
def gaussian_rows(N: int, d: int, seed: int, dtype: str = "fp32", outliers: int = 0,
                  outlier_scale: float = 10.0):
    """Generic small case for parity tests: N(0,1) rows with `outliers` scaled channels, stored
    as fp32 / fp16 / bf16 bits."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((N, d), dtype=np.float32)
    if outliers:
        ch = rng.permutation(d)[:outliers]
        X[:, ch] *= np.float32(outlier_scale)
    if dtype == "fp32":
        return X
    if dtype == "fp16":
        return X.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(X)
    raise ValueError(dtype)
