"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Packed codes must match bit for bit; a disagreement is tolerated only where the oracle
itself shows a decision within 1e-6 of its boundary (counted and printed).  Scores and outputs must
agree within 1e-3 (relative, as defined in gpu_util)."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import (cache_from_records, check_out, check_scores, gpu_decode, gpu_encode, new_cache,  # noqa: E402
                      record_gammas, score_floor)

ALL_BITS = (1, 1.5, 2, 2.5, 3, 4)


def make_inputs(seed, n_seq, n_kv, n_tok, d, dtype, sigma_ln=0.5, n_outlier=4):
    wl = synth.Workload("t", n_seq, n_kv, n_kv, d, n_tok, 3.0, dtype, sigma_ln=sigma_ln, n_outlier=n_outlier)
    keys = np.stack([np.stack([synth.keys_block(seed, wl, s, h, 0, n_tok) for h in range(n_kv)], axis=1)
                     for s in range(n_seq)])                                   # [n_seq, n_tok, n_kv, d]
    vals = np.stack([np.stack([synth.values_block(seed, wl, s, h, 0, n_tok) for h in range(n_kv)], axis=0)
                     for s in range(n_seq)])                                   # [n_seq, n_kv, n_tok, d]
    signs = synth.sign_vectors(seed, n_kv, d)
    return keys, vals, signs


# Caps on the boundary ties per triplet compared: a few times what a healthy encoder shows (about 1e-5 at full
# size; small cases may show a handful)
MAX_TIE_RATE = 5e-5
MAX_SCALED_ONLY_RATE = 2e-5


def compare_records(plan, keys, signs, rec, tag, max_ties=None, mode=oracle.MODE_LOCAL_3X3):
    """keys [n_seq, n_tok, n_kv, d]; rec [n_seq, n_kv, >= n_tok, rb] from the GPU; mode: the oracle's rounding mode.
    Returns (equal, ties under a plain 1e-6 on every compared quantity, ties only the l1-scaled reading admits,
    hard); max_ties: an explicit cap on all ties instead of the rate."""
    n_seq, n_tok, n_kv, d = keys.shape
    total = np.zeros(4, dtype=np.int64)
    for s in range(n_seq):
        for h in range(n_kv):
            k = keys[s, :, h, :].astype(np.float64)
            got = rec[s, h, :n_tok]
            ref = oracle.encode(plan, k, signs[h], mode=mode)
            g_got = got[:, :4].copy().view(np.float32)[:, 0].astype(np.float64)
            g_ref = ref[:, :4].copy().view(np.float32)[:, 0].astype(np.float64)
            assert np.all(np.abs(g_got - g_ref) <= 1e-6 * np.maximum(g_ref, 1e-30)), tag   # gamma: fp32 norm
            if np.array_equal(got[:, 4:], ref[:, 4:]):
                total[0] += n_tok * plan.n_tri
            else:
                total += np.array(oracle.classify_both(plan, k, signs[h], got, tol=1e-6, mode=mode))
    print(f"[codes] {tag}: triplets equal={total[0]} ties_literal_1e-6={total[1]} ties_scaled_only={total[2]} "
          f"hard={total[3]}")
    assert total[3] == 0, f"{tag}: {total[3]} code mismatches away from any decision boundary"
    ties = total[1] + total[2]
    if max_ties is not None:
        assert ties <= max_ties, f"{tag}: too many boundary ties ({ties})"
    else:
        # a tie needs a decision boundary within the rounding error of the fp32 path: their number grows with the
        # number of levels per octahedral coordinate (the rates above are those of up to 32 levels)
        levels = max(1 << bd for _, bd, _ in plan.classes)
        rate = MAX_TIE_RATE * max(1, levels // 32)
        assert ties <= max(3, rate * total.sum()), f"{tag}: too many boundary ties ({ties})"
        assert total[2] <= max(2, MAX_SCALED_ONLY_RATE * total.sum()), f"{tag}: too many scaled-only ties ({total[2]})"
    return total


# ---- encode ----------------------------------------------------------------------------------

def test_encode_tiny_config_fp32():
    """1 sequence, 1 KV head, d = 128, 4096 tokens, fp32 keys, 3 bits."""
    cb = binding.octopus_build_codebooks(128, 3)
    plan = oracle.make_plan(128, 3)
    wl = synth.WORKLOADS["tiny"]
    keys = synth.keys_block(1, wl, 0, 0, 0, wl.n_tokens)[None, :, None, :]
    signs = synth.sign_vectors(1, 1, 128)
    rec, pad, _ = gpu_encode(cb, keys, "fp32", signs, 4096)
    assert not pad.any()
    compare_records(plan, keys, signs, rec, "tiny fp32 b=3")


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("bits", ALL_BITS)
def test_encode_all_plans_bf16_ragged_tail(d, bits):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, _, signs = make_inputs(int(d + 10 * bits), 2, 2, 200, d, "bf16")     # 3 tiles + a tail of 8
    rec, pad, _ = gpu_encode(cb, keys, "bf16", signs, 256)
    assert not pad.any()
    assert not rec[:, :, 200:].any()                                          # untouched slots stay zero
    compare_records(plan, keys, signs, rec, f"d={d} b={bits}")


def test_encode_append_at_unaligned_positions_leaves_other_slots_alone():
    cb = binding.octopus_build_codebooks(128, 3)
    plan = oracle.make_plan(128, 3)
    keys, _, signs = make_inputs(5, 3, 2, 100, 128, "bf16")
    start = [0, 37, 150]
    cache = new_cache(cb, 3, 2, 256, fill=0xAB)
    rec, pad, _ = gpu_encode(cb, keys, "bf16", signs, 256, start_pos=start, cache=cache)
    for s, st in enumerate(start):
        hi = min(st + 100, 256)
        assert np.all(rec[s, :, :st] == 0xAB) and np.all(rec[s, :, hi:] == 0xAB)
        assert np.all(pad[s, :, :st] == 0xAB) and np.all(pad[s, :, hi:] == 0xAB)
        shifted = rec[s:s + 1, :, st:hi]
        compare_records(plan, keys[s:s + 1, :hi - st], signs, shifted, f"append at {st}")
    # streaming: one token per sequence per call reproduces the bulk result
    cache2 = new_cache(cb, 3, 2, 256, fill=0xAB)
    for t in range(3):
        gpu_encode(cb, keys[:, t:t + 1], "bf16", signs, 256, start_pos=[st + t for st in start], cache=cache2)
    from paper_2605_21226_amd import layout
    rec2, _ = layout.cache_to_records(cache2.cpu().numpy(), 3, 2, 256, cb.plan.granules, cb.plan.record_bytes)
    for s, st in enumerate(start):
        assert np.array_equal(rec2[s, :, st:st + 3], rec[s, :, st:st + 3])


def test_encode_degenerate_keys():
    """all-zero key, one-hot keys, a constant key, tiny and huge magnitudes.  Per key: the zero key's record is
    the oracle's placeholder byte for byte; scaling a key by a power of two changes gamma only, so those keys
    behave like any other; a one-hot or constant key rotates to coordinates of equal magnitude, where EVERY
    decision of Alg. 1 sits exactly on a boundary (p = (+-1/3, +-1/3, +-1/3), nine candidates with equal
    scores): any of its triplets may tie, none may be a hard mismatch."""
    d = 128
    cb = binding.octopus_build_codebooks(d, 3)
    plan = oracle.make_plan(d, 3)
    rng = np.random.default_rng(3)
    keys = synth.round_to_bf16(rng.standard_normal((1, 64, 1, d)).astype(np.float32))
    keys[0, 0, 0, :] = 0.0
    keys[0, 1, 0, :] = 0.0; keys[0, 1, 0, 5] = 1.0
    keys[0, 2, 0, :] = 0.0; keys[0, 2, 0, 127] = -3.0
    keys[0, 3, 0, :] *= np.float32(2.0 ** -60)
    keys[0, 4, 0, :] *= np.float32(2.0 ** 40)
    keys[0, 5, 0, :] = 1.0
    signs = synth.sign_vectors(3, 1, d)
    rec, _, _ = gpu_encode(cb, keys, "bf16", signs, 64)
    ref0 = oracle.encode(plan, np.zeros((1, d)), signs[0])[0]
    assert np.array_equal(rec[0, 0, 0], ref0)                                 # the zero key's placeholder
    symmetric = [1, 2, 5]                                                      # every decision on a boundary
    ordinary = [t for t in range(64) if t not in symmetric]
    for t in symmetric:
        compare_records(plan, keys[:, t:t + 1], signs, rec[:, :, t:t + 1], f"degenerate key {t}", max_ties=8)
    compare_records(plan, keys[:, ordinary], signs, rec[:, :, ordinary], "degenerate keys: the ordinary ones", max_ties=1)


# ---- decode attention ------------------------------------------------------------------------------

def oracle_attention_all(plan, records, signs, q, v, lens, scale):
    """records [n_seq, n_kv, T, rb], q [n_seq, n_q, n_qh, d], v [n_seq, n_kv, T, d]"""
    n_seq, n_q, n_qh, d = q.shape
    n_kv = v.shape[1]
    g = n_qh // n_kv
    out = np.zeros((n_seq, n_q, n_qh, d))
    scores = {}
    for s in range(n_seq):
        for h in range(n_kv):
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            L = int(lens[s])
            sc, o, gap = oracle.attention(plan, records[s, h, :L], signs[h], qq, v[s, h, :L].astype(np.float64), scale)
            assert gap < 1e-9
            out[s, :, h * g:(h + 1) * g, :] = o.reshape(n_q, g, d)
            scores[(s, h)] = sc.reshape(n_q, g, L)
    return out, scores


def run_decode_case(d, bits, n_seq, n_qh, n_kv, n_q, lens, dtype, seed, t_capacity=None, want_scores=True):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    T = max(int(max(lens)), 1)
    t_capacity = t_capacity or -(-T // 64) * 64
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, dtype)
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(n_seq)])
    wl = synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, dtype, n_q=n_q)
    q = synth.queries(seed, wl)
    v = np.zeros((n_seq, n_kv, t_capacity, d), dtype=np.float32)
    v[:, :, :T] = vals
    scale = 1.0 / np.sqrt(d)
    cache = cache_from_records(cb, records, t_capacity)      # the oracle's codes in the device layout
    out, scores = gpu_decode(cb, q, dtype, signs, cache, t_capacity, v, dtype, lens, scale, want_scores=want_scores)
    ref_out, ref_scores = oracle_attention_all(plan, records, signs, q, v, lens, scale)
    g = n_qh // n_kv
    worst_s = worst_o = 0.0
    for s in range(n_seq):
        L = int(lens[s])
        for h in range(n_qh):
            for qi in range(n_q):
                if L == 0:
                    assert np.all(out[s, qi, h] == 0.0)
                    continue
                if want_scores:
                    floor = score_floor(q[s, qi, h], record_gammas(records[s, h // g, :L]), scale)
                    worst_s = max(worst_s, check_scores(scores[s, qi, h, :L], ref_scores[(s, h // g)][qi, h % g], floor))
                worst_o = max(worst_o, check_out(out[s, qi, h], ref_out[s, qi, h]))
        if want_scores:
            assert np.all(np.isnan(scores[s, :, :, L:]))      # scores past len are not written
    print(f"[attn] d={d} b={bits} lens={list(lens)}: worst score err {worst_s:.3g} x tol, worst out err {worst_o:.3g}")


def test_decode_tiny_config_fp32():
    run_decode_case(128, 3, 1, 1, 1, 1, [4096], "fp32", seed=1)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_decode_gqa_ragged_d128(bits):
    run_decode_case(128, bits, 3, 8, 2, 1, [0, 77, 1000], "bf16", seed=int(10 * bits))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_decode_mha_multi_query_d64(bits):
    run_decode_case(64, bits, 1, 3, 3, 5, [700], "bf16", seed=int(100 + 10 * bits))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_decode_gqa2_ragged_d256(bits):
    run_decode_case(256, bits, 2, 4, 2, 1, [513, 64], "bf16", seed=int(200 + 10 * bits))


def test_decode_rows_not_a_power_of_two_and_many_row_groups():
    run_decode_case(128, 3, 1, 6, 2, 1, [300], "bf16", seed=7)       # 3 query heads per KV head
    run_decode_case(64, 4, 1, 2, 2, 11, [300], "bf16", seed=8)       # 11 query rows -> two groups of 8


@pytest.mark.parametrize("bits", ALL_BITS)
def test_decode_many_query_rows_d64(bits):
    """40 and 200 query rows per KV head (the matrix-core kernel: blocks of 128 rows), ragged lengths"""
    run_decode_case(64, bits, 2, 2, 2, 40, [700, 65], "bf16", seed=int(300 + 10 * bits), want_scores=False)
    if bits == 4:
        run_decode_case(64, bits, 1, 3, 3, 200, [1000], "bf16", seed=341, want_scores=False)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_decode_many_query_rows_gqa_d128(bits):
    """16 queries x 4 heads per KV head = 64 rows; a sequence of length 0 and a ragged last tile"""
    run_decode_case(128, bits, 3, 8, 2, 16, [0, 130, 513], "bf16", seed=int(400 + 10 * bits), want_scores=False)


def test_decode_many_query_rows_with_scores_or_fp32_values_uses_the_row_group_kernels():
    run_decode_case(64, 4, 1, 2, 2, 40, [300], "bf16", seed=351)                    # scores requested
    run_decode_case(64, 4, 1, 2, 2, 40, [300], "fp32", seed=352, want_scores=False)  # fp32 values


def test_decode_is_independent_of_the_split_count():
    d, bits, T = 128, 3, 8192
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, vals, signs = make_inputs(11, 1, 1, T, d, "bf16")
    records = oracle.encode(plan, keys[0, :, 0].astype(np.float64), signs[0])[None, None]
    q = synth.queries(11, synth.Workload("t", 1, 4, 1, d, T, bits, "bf16"))
    cache = cache_from_records(cb, records, T)
    scale = 1 / np.sqrt(d)
    a, _ = gpu_decode(cb, q, "bf16", signs, cache, T, vals, "bf16", [5000], scale, want_scores=False, max_len=5000)
    b, _ = gpu_decode(cb, q, "bf16", signs, cache, T, vals, "bf16", [5000], scale, want_scores=False, max_len=8192)
    assert np.max(np.abs(a - b)) <= 1e-5 * np.max(np.abs(a))
    again, _ = gpu_decode(cb, q, "bf16", signs, cache, T, vals, "bf16", [5000], scale, want_scores=False, max_len=5000)
    assert np.array_equal(a, again)                                   # run-to-run deterministic


def test_encode_then_decode_end_to_end():
    """GPU codes into GPU attention, against oracle codes into oracle attention."""
    d, bits, n_seq, n_qh, n_kv, T = 128, 3, 2, 8, 2, 1500
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, vals, signs = make_inputs(21, n_seq, n_kv, T, d, "bf16")
    cap = 1536
    _, _, cache = gpu_encode(cb, keys, "bf16", signs, cap)
    q = synth.queries(21, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16"))
    v = np.zeros((n_seq, n_kv, cap, d), dtype=np.float32)
    v[:, :, :T] = vals
    lens = [T, 901]
    scale = 1 / np.sqrt(d)
    out, _ = gpu_decode(cb, q, "bf16", signs, cache, cap, v, "bf16", lens, scale, want_scores=False)
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(n_seq)])
    ref_out, _ = oracle_attention_all(plan, records, signs, q, v, lens, scale)
    for s in range(n_seq):
        for h in range(n_qh):
            check_out(out[s, 0, h], ref_out[s, 0, h])


def test_decode_more_sequences_than_lanes():
    """70 short ragged sequences (some empty): the work plan is looked up by binary search beyond 63
    sequences, by one round of loads below."""
    rng = np.random.default_rng(12)
    lens = [int(x) for x in rng.integers(0, 400, size=70)]
    lens[3] = 0
    lens[69] = 399
    run_decode_case(64, 3, 70, 2, 1, 1, lens, "bf16", seed=501, want_scores=False)
    run_decode_case(64, 3, 63, 2, 1, 1, lens[:63], "bf16", seed=502, want_scores=False)
