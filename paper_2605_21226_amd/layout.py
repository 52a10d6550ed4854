"""Index arithmetic between canonical key records and the device cache layout
declared in include/octopus.h (no codec arithmetic here).

canonical: uint8 [n_seq, n_kv_heads, n_tokens, record_bytes]
device:    uint8 [n_seq, n_kv_heads, t_capacity / 64, granules, 64, 16]
           (byte x of token t at ((t // 64 * granules + x // 16) * 64 + t % 64) * 16 + x % 16)
"""
from __future__ import annotations

import numpy as np

TILE = 64


def records_to_cache(records, granules, t_capacity):
    """numpy uint8 canonical records -> numpy uint8 device image (flat)."""
    records = np.asarray(records, dtype=np.uint8)
    n_seq, n_kv, n_tok, rb = records.shape
    assert t_capacity % TILE == 0 and n_tok <= t_capacity and rb <= granules * 16
    padded = np.zeros((n_seq, n_kv, t_capacity, granules * 16), dtype=np.uint8)
    padded[:, :, :n_tok, :rb] = records
    tiles = padded.reshape(n_seq, n_kv, t_capacity // TILE, TILE, granules, 16)
    return np.ascontiguousarray(tiles.transpose(0, 1, 2, 4, 3, 5)).reshape(-1)


def cache_to_records(cache, n_seq, n_kv_heads, t_capacity, granules, record_bytes, n_tokens=None):
    """numpy uint8 device image -> canonical records [n_seq, n_kv_heads, n_tokens, record_bytes]
    and the padding bytes [.., granules * 16 - record_bytes] (which the encoder leaves zero)."""
    cache = np.asarray(cache, dtype=np.uint8).reshape(n_seq, n_kv_heads, t_capacity // TILE, granules, TILE, 16)
    rows = np.ascontiguousarray(cache.transpose(0, 1, 2, 4, 3, 5)).reshape(n_seq, n_kv_heads, t_capacity, granules * 16)
    n_tokens = t_capacity if n_tokens is None else n_tokens
    return rows[:, :, :n_tokens, :record_bytes].copy(), rows[:, :, :n_tokens, record_bytes:].copy()


def qjl_to_canonical(qjl, n_seq, n_kv_heads, t_capacity, head_dim):
    """numpy uint8 side-car image -> (sign bits uint8 [n_seq, n_kv_heads, t_capacity, d/8], bit j%8 of byte j/8
    set when sigma_j = -1; gamma_r float16 [n_seq, n_kv_heads, t_capacity])."""
    nw = head_dim // 32
    tq = TILE * (head_dim // 8 + 2)
    img = np.asarray(qjl, dtype=np.uint8).reshape(n_seq, n_kv_heads, t_capacity // TILE, tq)
    words = np.ascontiguousarray(img[..., :nw * TILE * 4]).view(np.uint32).reshape(n_seq, n_kv_heads, t_capacity // TILE,
                                                                                   nw, TILE)
    words = np.ascontiguousarray(words.transpose(0, 1, 2, 4, 3)).reshape(n_seq, n_kv_heads, t_capacity, nw)
    bits = words.view(np.uint8).reshape(n_seq, n_kv_heads, t_capacity, nw * 4)
    gamma_r = np.ascontiguousarray(img[..., nw * TILE * 4:]).view(np.float16).reshape(n_seq, n_kv_heads, t_capacity)
    return bits, gamma_r


def qjl_from_canonical(bits, gamma_r, t_capacity):
    """Inverse of qjl_to_canonical: sign bits uint8 [n_seq, n_kv_heads, n_tokens, d/8] and gamma_r float16
    [n_seq, n_kv_heads, n_tokens] -> numpy uint8 side-car image for t_capacity tokens (other slots zero)."""
    bits = np.asarray(bits, dtype=np.uint8)
    n_seq, n_kv, n_tok, nb = bits.shape
    nw = nb // 4
    full = np.zeros((n_seq, n_kv, t_capacity, nb), dtype=np.uint8)
    full[:, :, :n_tok] = bits
    g = np.zeros((n_seq, n_kv, t_capacity), dtype=np.float16)
    g[:, :, :n_tok] = np.asarray(gamma_r, dtype=np.float16)
    words = full.view(np.uint32).reshape(n_seq, n_kv, t_capacity // TILE, TILE, nw).transpose(0, 1, 2, 4, 3)
    img = np.concatenate([np.ascontiguousarray(words).view(np.uint8).reshape(n_seq, n_kv, t_capacity // TILE, -1),
                          g.reshape(n_seq, n_kv, t_capacity // TILE, TILE).view(np.uint8)], axis=-1)
    return np.ascontiguousarray(img).reshape(-1)
