"""Seeded synthetic inputs generated directly in device memory, for workloads too large to draw on
the host (several GB of keys and values).  Same recipe as paper_2605_21226_amd.synth: per-channel
log-normal scales with outlier channels for the keys, N(0, 1) values and queries, rounded to the
workload's dtype.  No codec arithmetic here; the oracle side of a test reads these tensors back.
"""
from __future__ import annotations

import numpy as np

from . import synth


def device_inputs(wl, seed, dev):
    """-> keys [n_seq, n_tokens, n_kv, d], vals [n_seq, n_kv, n_tokens, d], q [n_seq, n_q, n_qh, d]
    (device tensors of the workload's dtype), signs [n_kv, d] (+-1, host), lens [n_seq] (int32, host)."""
    import torch

    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    sig = torch.from_numpy(synth.channel_scales(seed, wl).astype(np.float32)).to(dev)       # [n_kv, d]
    keys = torch.empty((wl.n_seq, wl.n_tokens, wl.n_kv_heads, wl.head_dim), dtype=dt, device=dev)
    vals = torch.empty((wl.n_seq, wl.n_kv_heads, wl.n_tokens, wl.head_dim), dtype=dt, device=dev)
    chunk = 4096
    for s in range(wl.n_seq):
        for t0 in range(0, wl.n_tokens, chunk):
            n = min(chunk, wl.n_tokens - t0)
            z = torch.randn((n, wl.n_kv_heads, wl.head_dim), generator=gen, device=dev)
            keys[s, t0:t0 + n] = (z * sig[None]).to(dt)
            z = torch.randn((wl.n_kv_heads, n, wl.head_dim), generator=gen, device=dev)
            vals[s, :, t0:t0 + n] = z.to(dt)
    q = torch.randn((wl.n_seq, wl.n_q, wl.n_q_heads, wl.head_dim), generator=gen, device=dev).to(dt)
    signs = synth.sign_vectors(seed, wl.n_kv_heads, wl.head_dim)
    lens = synth.context_lengths(seed, wl)
    return keys, vals, q, signs, lens
