"""Pins of the oracle's hybrid-cache attention (compressed tokens + a native-precision window)."""
import numpy as np
import scipy.special

import oracle
from paper_2605_21226_amd import synth


def _case(seed, n, w, d=128, bits=3, n_q=3):
    rng = np.random.default_rng(seed)
    plan = oracle.make_plan(d, bits)
    s = synth.sign_vectors(seed, 1, d)[0]
    keys = rng.standard_normal((n + w, d)) * 1.5
    v = rng.standard_normal((n + w, d))
    q = rng.standard_normal((n_q, d))
    rec = oracle.encode(plan, keys[:n], s)
    return plan, s, keys, v, q, rec


def test_empty_window_is_the_plain_compressed_attention():
    plan, s, keys, v, q, rec = _case(1, 200, 0)
    sc, out = oracle.attention_hybrid(plan, rec, s, np.zeros((0, 128)), q, v, 0.1)
    ref_sc, ref_out, _ = oracle.attention(plan, rec, s, q, v, 0.1)
    assert np.allclose(sc, ref_sc, atol=1e-12) and np.allclose(out, ref_out, atol=1e-12)


def test_nothing_compressed_is_textbook_attention():
    plan, s, keys, v, q, rec = _case(2, 0, 40)
    sc, out = oracle.attention_hybrid(plan, rec, s, keys, q, v, 0.09)
    assert np.allclose(sc, 0.09 * q @ keys.T, atol=1e-12)
    assert np.allclose(out, scipy.special.softmax(0.09 * q @ keys.T, axis=1) @ v, atol=1e-12)


def test_window_scores_are_exact_and_parts_merge_by_the_flash_decoding_identity():
    """App. A: the two parts, each with its own (m, l, acc), combine into the whole."""
    plan, s, keys, v, q, rec = _case(3, 300, 32)
    sc, out = oracle.attention_hybrid(plan, rec, s, keys[300:], q, v, 0.1)
    assert np.allclose(sc[:, 300:], 0.1 * q @ keys[300:].T, atol=1e-12)            # window: the true keys
    sc_c, out_c, _ = oracle.attention(plan, rec, s, q, v[:300], 0.1)
    assert np.allclose(sc[:, :300], sc_c, atol=1e-12)
    m_c, m_w = sc_c.max(axis=1), sc[:, 300:].max(axis=1)
    l_c, l_w = np.exp(sc_c - m_c[:, None]).sum(axis=1), np.exp(sc[:, 300:] - m_w[:, None]).sum(axis=1)
    out_w = scipy.special.softmax(sc[:, 300:], axis=1) @ v[300:]
    m = np.maximum(m_c, m_w)
    a, b = np.exp(m_c - m) * l_c, np.exp(m_w - m) * l_w
    merged = (a[:, None] * out_c + b[:, None] * out_w) / (a + b)[:, None]
    assert np.allclose(out, merged, atol=1e-12)
    # keeping recent tokens exact moves the result towards uncompressed attention
    exact = scipy.special.softmax(0.1 * q @ keys.T, axis=1) @ v
    all_c = oracle.attention(plan, oracle.encode(plan, keys, s), s, q, v, 0.1)[1]
    assert np.linalg.norm(out - exact) < np.linalg.norm(all_c - exact)
