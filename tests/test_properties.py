"""Property tests (hypothesis) of the index arithmetic between canonical records and the device layouts,
and of the oracle's stream packing: round trips for arbitrary shapes and contents."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from paper_2605_21226_amd import layout

SETTINGS = dict(max_examples=40, deadline=None)


@settings(**SETTINGS)
@given(n_seq=st.integers(1, 3), n_kv=st.integers(1, 3), tiles=st.integers(1, 4), n_tok=st.integers(0, 256),
       granules=st.integers(1, 10), slack=st.integers(0, 15), seed=st.integers(0, 2 ** 31 - 1))
def test_cache_layout_round_trip(n_seq, n_kv, tiles, n_tok, granules, slack, seed):
    cap = 64 * tiles
    n_tok = min(n_tok, cap)
    rb = max(granules * 16 - slack, 5)
    rec = np.random.default_rng(seed).integers(0, 256, (n_seq, n_kv, n_tok, rb), dtype=np.uint8)
    img = layout.records_to_cache(rec, granules, cap)
    assert img.size == n_seq * n_kv * cap * granules * 16
    back, pad = layout.cache_to_records(img, n_seq, n_kv, cap, granules, rb)
    assert np.array_equal(back[:, :, :n_tok], rec) and not back[:, :, n_tok:].any() and not pad.any()
    # byte x of the record of token t sits where the header says
    if n_tok:
        t, x = n_tok - 1, rb - 1
        off = ((t // 64 * granules + x // 16) * 64 + t % 64) * 16 + x % 16
        region = img.reshape(n_seq, n_kv, -1)[0, 0]
        assert region[off] == rec[0, 0, t, x]


@settings(**SETTINGS)
@given(d=st.sampled_from([64, 128, 256]), n_tok=st.integers(1, 200), seed=st.integers(0, 2 ** 31 - 1))
def test_qjl_layout_round_trip(d, n_tok, seed):
    rng = np.random.default_rng(seed)
    cap = -(-n_tok // 64) * 64
    bits = rng.integers(0, 256, (2, 2, n_tok, d // 8), dtype=np.uint8)
    g = rng.random((2, 2, n_tok)).astype(np.float16)
    img = layout.qjl_from_canonical(bits, g, cap)
    assert img.size == 2 * 2 * cap * (d // 8 + 2)
    b2, g2 = layout.qjl_to_canonical(img, 2, 2, cap, d)
    assert np.array_equal(b2[:, :, :n_tok], bits) and np.array_equal(g2[:, :, :n_tok], g)


@settings(**SETTINGS)
@given(d=st.sampled_from([64, 128, 256]), bits=st.sampled_from([1, 1.5, 2, 2.5, 3, 4]), seed=st.integers(0, 2 ** 31 - 1))
def test_oracle_pack_unpack_round_trip(d, bits, seed):
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(seed)
    n_tri = plan.n_tri
    idx_dir = np.zeros(2 * n_tri, dtype=np.int32)
    idx_nrm = np.zeros(n_tri, dtype=np.int32)
    pos = 0
    for n, b_dir, b_nrm in plan.classes:
        idx_dir[2 * pos:2 * (pos + n)] = rng.integers(0, 1 << b_dir, 2 * n)
        idx_nrm[pos:pos + n] = rng.integers(0, 1 << b_nrm, n)
        pos += n
    gamma = float(np.float32(rng.random() * 10))
    rec = oracle.pack_record(plan, gamma, idx_dir, idx_nrm)
    assert rec.shape == (plan.record_bytes,)
    g2, d2, n2 = oracle.unpack_record(plan, rec)
    assert g2 == gamma and np.array_equal(d2, idx_dir) and np.array_equal(n2, idx_nrm)


@settings(**SETTINGS)
@given(bits=st.sampled_from([2, 3, 4]), group=st.sampled_from([16, 32]), d=st.sampled_from([64, 128]),
       seed=st.integers(0, 2 ** 31 - 1), scale=st.sampled_from([1e-20, 1e-3, 1.0, 1e6, 1e30]))
def test_value_codec_error_bound_for_any_magnitude(bits, group, d, seed, scale):
    v = (np.random.default_rng(seed).standard_normal((5, d)) * scale).astype(np.float32)
    rows = oracle.vq_encode(v, bits, group)
    v_hat = oracle.vq_decode(rows, d, bits, group)
    vg = v.reshape(5, d // group, group).astype(np.float64)
    step = (vg.max(axis=2) - vg.min(axis=2)) / (2 ** bits - 1)
    err = np.abs(v_hat.reshape(5, d // group, group) - vg)
    assert np.all(err <= 0.5 * step[:, :, None] * (1 + 1e-5) + 1e-45)
