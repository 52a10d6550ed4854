"""Seeded synthetic inputs shaped like KV caches of text, video and audio decoders.

This module holds no arithmetic of the codec: it only draws random numbers.
It is the one module that both the HIP path's tests / benchmark and the CPU
oracle's tests use, so that both sides see the same inputs.

Recipe (per KV head): key[t, c] = sigma_c * z[t, c] with z ~ N(0, 1),
sigma_c ~ LogNormal(0, sigma_ln) drawn once per (head, channel), and
`n_outlier` channels per head scaled by `outlier_scale` (the heavy channels
real decoder keys show).  Queries and values are N(0, 1).  Where a workload
says bf16 the values are rounded to bf16 (round to nearest even) and both
sides consume those rounded numbers.  WHT sign vectors are uniform +-1.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n_seq: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_tokens: int          # cached tokens per sequence (max when ragged)
    bits: float            # nominal bits / coordinate
    dtype: str             # "fp32" or "bf16"
    sigma_ln: float = 0.5
    n_outlier: int = 4
    outlier_scale: float = 10.0
    n_q: int = 1           # queries per sequence in one decode call
    ragged_min: int = 0    # > 0: context lengths uniform in [ragged_min, n_tokens]
    n_new: int = 0         # tokens encoded in the timed encode leg


# The five workloads named by the build's baseline configuration.
WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 1, 128, 4096, 3.0, "fp32", n_new=4096),
    "llama3_8b_decode": Workload("llama3_8b_decode", 16, 32, 8, 128, 32768, 3.0, "bf16", n_new=32768),
    "long_context_2bit": Workload("long_context_2bit", 4, 32, 8, 128, 131072, 2.0, "bf16", n_new=1),
    "causal_video": Workload("causal_video", 1, 24, 24, 64, 75600, 4.0, "bf16", sigma_ln=0.3, n_outlier=0,
                             n_q=3600, n_new=3600),
    "ragged_d256": Workload("ragged_d256", 32, 16, 8, 256, 65536, 3.0, "bf16", ragged_min=1024, n_new=65536),
}


def round_to_bf16(x):
    """Round fp32 values to the nearest bf16 (ties to even); returns fp32 holding bf16 values."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(x):
    """uint16 bit patterns of values already representable in bf16."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def _rng(seed, *stream):
    return np.random.default_rng([int(seed)] + [int(s) for s in stream])


def sign_vectors(seed, n_kv_heads, head_dim):
    """[n_kv_heads, head_dim] int8 of +-1, one vector per KV head."""
    r = _rng(seed, 101)
    return (r.integers(0, 2, size=(n_kv_heads, head_dim)).astype(np.int8) * 2 - 1)


def sign_bits(signs_pm1):
    """Pack +-1 sign vectors into bytes, bit j of byte j // 8 set when s_j = -1 (LSB first)."""
    neg = (np.asarray(signs_pm1) < 0).astype(np.uint8)
    return np.packbits(neg, axis=-1, bitorder="little")


def channel_scales(seed, wl: Workload):
    """[n_kv_heads, head_dim] per-channel standard deviations."""
    r = _rng(seed, 202)
    sig = np.exp(wl.sigma_ln * r.standard_normal((wl.n_kv_heads, wl.head_dim)))
    for h in range(wl.n_kv_heads):
        if wl.n_outlier > 0:
            ch = r.choice(wl.head_dim, size=wl.n_outlier, replace=False)
            sig[h, ch] *= wl.outlier_scale
    return sig


def _maybe_bf16(x, dtype):
    x = x.astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def keys_block(seed, wl: Workload, seq, head, t0, n):
    """keys of tokens [t0, t0 + n) of (seq, head): fp32 array [n, head_dim]
    (holding bf16-representable values when wl.dtype is bf16)."""
    sig = channel_scales(seed, wl)[head]
    z = _rng(seed, 303, seq, head, t0).standard_normal((n, wl.head_dim))
    return _maybe_bf16(z * sig[None, :], wl.dtype)


def values_block(seed, wl: Workload, seq, head, t0, n):
    z = _rng(seed, 404, seq, head, t0).standard_normal((n, wl.head_dim))
    return _maybe_bf16(z, wl.dtype)


def queries(seed, wl: Workload):
    """[n_seq, n_q, n_q_heads, head_dim]"""
    z = _rng(seed, 505).standard_normal((wl.n_seq, wl.n_q, wl.n_q_heads, wl.head_dim))
    return _maybe_bf16(z, wl.dtype)


def context_lengths(seed, wl: Workload):
    """[n_seq] int32 context lengths (all n_tokens unless the workload is ragged)."""
    if wl.ragged_min <= 0:
        return np.full(wl.n_seq, wl.n_tokens, dtype=np.int32)
    r = _rng(seed, 606)
    return r.integers(wl.ragged_min, wl.n_tokens + 1, size=wl.n_seq).astype(np.int32)


def gaussian_keys(seed, n, head_dim):
    """Isotropic N(0, 1) keys, the synthetic probe of the paper's rate-quality tables."""
    return _rng(seed, 707).standard_normal((n, head_dim))


def gaussian_queries(seed, n, head_dim):
    return _rng(seed, 808).standard_normal((n, head_dim))
