"""Pins of the oracle's value codec (per-group uniform quantisation).  The paper fixes only the group
size, the bit width and the byte count; the rest is a reading (parity unpinned by the paper), pinned here
to what the mathematics of a uniform quantiser fixes."""
import numpy as np
import pytest

import oracle


def _vals(seed, n, d):
    rng = np.random.default_rng(seed)
    v = rng.standard_normal((n, d)).astype(np.float32)
    return (v.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)      # bf16-representable, as the workloads'


def _fields(rows, d, bits, group):
    """codes [n, d] and (scale, zero) [n, d/group] read back with numpy only"""
    nb = bits * d // 8
    bitsarr = np.unpackbits(rows[:, :nb], axis=1, bitorder="little").reshape(rows.shape[0], d, bits)
    codes = (bitsarr.astype(np.int64) << np.arange(bits)).sum(axis=2)
    meta = np.ascontiguousarray(rows[:, nb:]).view(np.float32).reshape(rows.shape[0], d // group, 2)
    return codes, meta[:, :, 0], meta[:, :, 1]


def test_row_bytes_are_the_ones_the_printed_kv_ratios_imply(golden):
    """Table (kernel speed): KV ratio = 4 d / (key record + value row) with the value row b d / 8 + 8 d / g."""
    for workload, d, g, b, ratio in golden("kv_ratio.txt"):
        d, g, b = int(d), int(g), int(b)
        plan = oracle.make_plan(d, b)
        assert round(4.0 * d / (plan.record_bytes + oracle.vq_row_bytes(d, b, g)), 1) == float(ratio)
    assert oracle.vq_row_bytes(128, 3, 32) == 48 + 32 and oracle.vq_row_bytes(64, 4, 16) == 32 + 32


def test_hand_example():
    # one group of 16 at 2 bits: lo = 0, hi = 3 -> scale 1; codes are the nearest integers, ties to even
    v = np.array([[0, 3, 1, 2, 0.4, 0.6, 0.5, 1.5, 2.5, 2.4, 2.6, 0, 0, 0, 0, 0]], dtype=np.float32)
    rows = oracle.vq_encode(v, 2, 16)
    codes, scale, zero = _fields(rows, 16, 2, 16)
    assert scale[0, 0] == 1.0 and zero[0, 0] == 0.0
    assert codes[0].tolist() == [0, 3, 1, 2, 0, 1, 0, 2, 2, 2, 3, 0, 0, 0, 0, 0]
    assert np.array_equal(oracle.vq_decode(rows, 16, 2, 16)[0], codes[0].astype(np.float64))
    # LSB-first: channel 0 in bits 0-1 of byte 0, channel 1 in bits 2-3, ...
    assert rows[0, 0] == (0 | 3 << 2 | 1 << 4 | 2 << 6)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [16, 32])
def test_codes_are_the_nearest_levels_and_errors_stay_within_half_a_step(bits, group):
    d, n = 128, 64
    v = _vals(bits * 10 + group, n, d)
    rows = oracle.vq_encode(v, bits, group)
    codes, scale, zero = _fields(rows, d, bits, group)
    v_hat = oracle.vq_decode(rows, d, bits, group)
    vg = v.reshape(n, d // group, group).astype(np.float64)
    # metadata: zero = group minimum exactly; scale = (max - min) / levels to fp32 rounding
    assert np.array_equal(zero, vg.min(axis=2).astype(np.float32))
    levels = 2 ** bits - 1
    assert np.allclose(scale, (vg.max(axis=2) - vg.min(axis=2)) / levels, rtol=3e-7, atol=0)
    # brute force over all levels: the stored code is the level nearest to the value (up to fp32 rounding ties)
    lv = zero[:, :, None, None].astype(np.float64) + scale[:, :, None, None].astype(np.float64) * np.arange(levels + 1)
    dist = np.abs(vg[:, :, :, None] - lv)                                   # [n, groups, g, levels]
    cg = codes.reshape(n, d // group, group)
    chosen = np.take_along_axis(dist, cg[..., None], axis=3)[..., 0]
    assert np.all(chosen <= dist.min(axis=3) + 1e-6 * scale[:, :, None])
    # reconstruction error at most half a step (plus rounding), extremes reproduced
    err = np.abs(v_hat.reshape(n, d // group, group) - vg)
    assert np.all(err <= 0.5 * scale[:, :, None] * (1 + 1e-6))
    assert np.all(cg.min(axis=2) == 0) and np.all(cg.max(axis=2) == levels)
    # decode is zero + scale * code exactly
    assert np.array_equal(v_hat.reshape(n, d // group, group),
                          zero[:, :, None].astype(np.float64) + scale[:, :, None].astype(np.float64) * cg)


def test_constant_group_and_packing_against_numpy():
    d, bits, group = 64, 3, 16
    v = _vals(3, 8, d)
    v[0, 16:32] = 1.25                                  # a constant group: scale 0, codes 0, exact
    rows = oracle.vq_encode(v, bits, group)
    codes, scale, zero = _fields(rows, d, bits, group)
    assert scale[0, 1] == 0.0 and zero[0, 1] == 1.25 and not codes[0, 16:32].any()
    assert np.all(oracle.vq_decode(rows, d, bits, group)[0, 16:32] == 1.25)
    # the code stream is numpy's little-endian bit packing of the codes, channel after channel
    bits_ref = ((codes[:, :, None] >> np.arange(bits)) & 1).astype(np.uint8).reshape(8, d * bits)
    assert np.array_equal(np.packbits(bits_ref, axis=1, bitorder="little"), rows[:, :bits * d // 8])


def test_more_bits_give_less_error_and_the_uniform_quantiser_noise_level():
    """For a uniform quantiser with step s the error is close to uniform on [-s/2, s/2]: variance s^2 / 12."""
    d, n, group = 128, 512, 32
    v = _vals(9, n, d)
    mse = {}
    for bits in (2, 3, 4):
        rows = oracle.vq_encode(v, bits, group)
        _, scale, _ = _fields(rows, d, bits, group)
        e = oracle.vq_decode(rows, d, bits, group) - v
        mse[bits] = float(np.mean(e ** 2))
        pred = float(np.mean(scale.astype(np.float64) ** 2) / 12.0)
        assert abs(mse[bits] - pred) <= (0.25 if bits == 2 else 0.1) * pred, (bits, mse[bits], pred)
    assert mse[4] < mse[3] < mse[2]
