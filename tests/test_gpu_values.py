"""GPU parity of the value codec (per-group quantised values): octopus_encode_values against the oracle's
rows byte for byte (every decision is a correctly rounded fp32 operation on both sides), and
octopus_attn_decode_vq against the oracle's attention over the dequantised rows (1e-3 bar of the plain
decoder)."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import (DEV, cache_from_records, check_out, check_scores, record_gammas, score_floor,  # noqa: E402
                      sign_bits_dev, to_dev)
from test_gpu_parity import make_inputs  # noqa: E402


def gpu_encode_values(vals, dtype, bits, group, cap, start_pos=None, fill=0):
    """vals numpy [n_seq, n_kv, n_tok, d] -> rows numpy [n_seq, n_kv, cap, row_bytes], device buffer"""
    n_seq, n_kv, n_tok, d = vals.shape
    rb = binding.octopus_vq_row_bytes(d, bits, group)
    vq = torch.full((binding.octopus_vq_bytes(d, bits, group, n_seq, n_kv, cap),), fill, dtype=torch.uint8, device=DEV)
    v_dev = to_dev(vals, dtype).permute(0, 2, 1, 3)              # [n_seq, n_tok, n_kv, d] view: strided input
    sp = None if start_pos is None else torch.tensor(start_pos, dtype=torch.int32, device=DEV)
    binding.octopus_encode_values(v_dev, bits, group, vq, cap, sp)
    torch.cuda.synchronize()
    return vq.cpu().numpy().reshape(n_seq, n_kv, cap, rb), vq


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [16, 32])
def test_encode_values_matches_the_oracle_byte_for_byte(d, bits, group):
    _, vals, _ = make_inputs(int(d + 10 * bits + group), 2, 2, 200, d, "bf16")
    rows, _ = gpu_encode_values(vals, "bf16", bits, group, 256)
    assert rows.shape[-1] == oracle.vq_row_bytes(d, bits, group)
    for s in range(2):
        for h in range(2):
            ref = oracle.vq_encode(vals[s, h], bits, group)
            assert np.array_equal(rows[s, h, :200], ref), (s, h)
    assert not rows[:, :, 200:].any()                                       # untouched rows stay as they were


def test_encode_values_fp32_append_and_degenerate_groups():
    d, bits, group = 128, 3, 32
    rng = np.random.default_rng(5)
    vals = rng.standard_normal((2, 1, 70, d)).astype(np.float32) * 3.0       # full fp32 mantissas
    vals[0, 0, 0, :32] = 0.75                                                # constant group
    vals[0, 0, 1, :] = 0.0                                                   # all-zero row
    vals[1, 0, 2, 5] = 1e30                                                  # one huge outlier
    vals[1, 0, 3, :] *= np.float32(1e-30)                                    # tiny magnitudes
    start = [0, 100]
    rows, _ = gpu_encode_values(vals, "fp32", bits, group, 192, start_pos=start, fill=0xEE)
    for s, st in enumerate(start):
        assert np.array_equal(rows[s, 0, st:st + 70], oracle.vq_encode(vals[s, 0], bits, group)), s
        assert np.all(rows[s, 0, :st] == 0xEE) and np.all(rows[s, 0, st + 70:] == 0xEE)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [16, 32])
def test_encode_values_quotients_at_half_integers_and_extreme_scales(bits, group):
    """(v - min) / scale exactly on, and one fp32 step beside, every half-integer, for scales whose reciprocal is
    not a power of two; then the same at scales near the ends of the fp32 range: the codes are the rounding (ties
    to even) of the correctly rounded quotient, whatever shortcut the kernel takes to it."""
    d, levels = 128, (1 << bits) - 1
    rng = np.random.default_rng(100 * bits + group)
    rows_in = []
    for scale in (3.0, 0.7, 1.0 / 3.0, 5.0e-3, 11.0, 1.0e-36, 2.0e-38, 3.0e36, 1.0e-41):
        sc = np.float32(scale)
        for _ in range(6):
            row = np.empty(d, dtype=np.float32)
            for g0 in range(0, d, group):
                k = rng.integers(0, levels, size=group).astype(np.float32) + np.float32(0.5)
                vals = (k * sc).astype(np.float32)
                step = rng.integers(-1, 2, size=group)                      # exactly on the tie, or one step off
                vals = np.where(step < 0, np.nextafter(vals, np.float32(0)), np.where(step > 0, np.nextafter(vals, np.float32(np.inf)), vals))
                vals[0], vals[1] = 0.0, np.float32(levels) * sc             # pins min and max of the group
                row[g0:g0 + group] = vals.astype(np.float32)
            rows_in.append(row)
    vals = np.stack(rows_in)[None, None]                                     # [1, 1, n_tok, d]
    n_tok = vals.shape[2]
    rows, _ = gpu_encode_values(vals, "fp32", bits, group, 64 * ((n_tok + 63) // 64))
    ref = oracle.vq_encode(vals[0, 0], bits, group)
    assert np.array_equal(rows[0, 0, :n_tok], ref)
    # the construction does hit ties: some group has quotients that are exact half-integers
    q = vals[0, 0, :6, :group] / ((vals[0, 0, :6, :group].max(axis=1, keepdims=True)) / np.float32(levels))
    assert np.any(np.abs(q - np.floor(q) - 0.5) == 0)


def test_encode_values_first_extreme_decides_the_sign_of_a_zero():
    """The stored minimum is the FIRST element that attains it (the scan of the codec's definition): with both
    zeros in a group, which one comes first shows in the sign bit of the stored zero point."""
    d, bits, group = 64, 3, 16
    rng = np.random.default_rng(9)
    rows_in = []
    for first, second in ((-0.0, 0.0), (0.0, -0.0)):
        for sign in (1.0, -1.0):                                  # zero is the minimum / the maximum of the group
            for _ in range(4):
                row = (np.abs(rng.standard_normal(d)) * sign).astype(np.float32)
                for g0 in range(0, d, group):
                    i, j = sorted(rng.choice(group, size=2, replace=False))
                    row[g0 + i], row[g0 + j] = first, second
                rows_in.append(row)
    rows_in.append(np.full(d, -0.0, dtype=np.float32))
    rows_in.append(np.zeros(d, dtype=np.float32))
    mixed = np.zeros(d, dtype=np.float32); mixed[::3] = -0.0
    rows_in.append(mixed)
    vals = np.stack(rows_in)[None, None]
    n_tok = vals.shape[2]
    for dtype in ("fp32", "bf16"):
        if dtype == "bf16":                                       # the same rows at the precision the kernel is handed
            vals = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
        rows, _ = gpu_encode_values(vals, dtype, bits, group, 64)
        assert np.array_equal(rows[0, 0, :n_tok], oracle.vq_encode(vals[0, 0], bits, group)), dtype
    # the fixture does what it says: stored minima of both signs occur
    ref = oracle.vq_encode(vals[0, 0], bits, group)
    zero_points = ref[:, bits * d // 8:].copy().view(np.float32)[:, 1::2]
    assert np.any(np.signbit(zero_points) & (zero_points == 0)) and np.any(~np.signbit(zero_points) & (zero_points == 0))


def run_decode_vq_case(d, bits, v_bits, group, n_seq, n_qh, n_kv, n_q, lens, seed, want_scores=True):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    T = max(int(max(lens)), 1)
    cap = -(-T // 64) * 64
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(n_seq)])
    rb = oracle.vq_row_bytes(d, v_bits, group)
    vq_rows = np.zeros((n_seq, n_kv, cap, rb), dtype=np.uint8)
    for s in range(n_seq):
        for h in range(n_kv):
            vq_rows[s, h, :T] = oracle.vq_encode(vals[s, h], v_bits, group)      # the oracle's rows, device layout
    wl = synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16", n_q=n_q)
    q = synth.queries(seed, wl)
    scale = 1.0 / np.sqrt(d)
    cache = cache_from_records(cb, records, cap)
    vq = torch.from_numpy(vq_rows.reshape(-1)).to(DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, T), dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    scores = (torch.full((n_seq, n_q, n_qh, cap), float("nan"), dtype=torch.float32, device=DEV) if want_scores else None)
    lens_dev = torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV)
    binding.octopus_attn_decode_vq(cb, to_dev(q, "bf16"), sign_bits_dev(signs), cache, cap, vq, v_bits, group, n_kv,
                                   lens_dev, T, scale, out, ws, scores)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    scores = scores.cpu().numpy() if want_scores else None
    g = n_qh // n_kv
    worst_s = worst_o = 0.0
    for s in range(n_seq):
        L = int(lens[s])
        for h in range(n_kv):
            if L == 0:
                assert np.all(out[s, :, h * g:(h + 1) * g] == 0.0)
                continue
            v_hat = oracle.vq_decode(vq_rows[s, h, :L], d, v_bits, group)
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            ref_s, ref_o, _ = oracle.attention(plan, records[s, h, :L], signs[h], qq, v_hat, scale)
            plain_o = oracle.attention(plan, records[s, h, :L], signs[h], qq, vals[s, h, :L].astype(np.float64), scale)[1]
            assert np.max(np.abs(plain_o - ref_o)) > 1e-3 * np.max(np.abs(ref_o))   # quantisation is visible at this bar
            ref_s, ref_o = ref_s.reshape(n_q, g, L), ref_o.reshape(n_q, g, d)
            for qi in range(n_q):
                for j in range(g):
                    if want_scores:
                        floor = score_floor(q[s, qi, h * g + j], record_gammas(records[s, h, :L]), scale)
                        worst_s = max(worst_s, check_scores(scores[s, qi, h * g + j, :L], ref_s[qi, j], floor))
                    worst_o = max(worst_o, check_out(out[s, qi, h * g + j], ref_o[qi, j]))
    print(f"[attn-vq] d={d} b={bits} v_bits={v_bits} g={group} lens={list(lens)}: worst score err {worst_s:.3g} x tol, "
          f"worst out err {worst_o:.3g}")


# Without score output the call is served by the matrix-core kernel (where one is built for the shape), with
# it by the kernel that multiplies on the vector units: both are held to the same bar.
@pytest.mark.parametrize("want_scores", [True, False])
@pytest.mark.parametrize("v_bits", [2, 3, 4])
@pytest.mark.parametrize("group", [16, 32])
def test_decode_vq_gqa_ragged_d128(v_bits, group, want_scores):
    run_decode_vq_case(128, 3, v_bits, group, 3, 8, 2, 1, [0, 77, 1000], seed=1100 + 10 * v_bits + group,
                       want_scores=want_scores)


@pytest.mark.parametrize("d,bits,v_bits,group", [(64, 4, 4, 16), (64, 2, 2, 32), (256, 2.5, 3, 32), (256, 3, 3, 16),
                                                 (128, 1.5, 2, 16)])
@pytest.mark.parametrize("want_scores", [True, False])
def test_decode_vq_other_shapes(d, bits, v_bits, group, want_scores):
    run_decode_vq_case(d, bits, v_bits, group, 2, 4, 2, 3, [513, 64], seed=int(1200 + d + 10 * bits),
                       want_scores=want_scores)


# Row groups of the matrix-core kernel: 1, 2 and 3 query rows per KV head ride in a group of four, 5 to 8 in a
# group of eight, more in several groups; every head dimension, code width and group size it is built for.
@pytest.mark.parametrize("d,bits,v_bits,group,n_qh,n_kv,n_q", [
    (128, 3, 3, 32, 2, 2, 1), (128, 2, 2, 32, 4, 2, 1), (128, 4, 4, 16, 3, 1, 1), (128, 2.5, 3, 16, 8, 1, 1),
    (128, 1, 4, 32, 4, 1, 3), (64, 3, 3, 32, 4, 1, 1), (64, 1.5, 2, 16, 8, 1, 2), (64, 4, 4, 32, 2, 2, 1),
    (256, 3, 3, 32, 4, 1, 1), (256, 2, 4, 32, 8, 2, 1), (256, 4, 2, 16, 4, 1, 1), (256, 1.5, 2, 32, 8, 1, 1),
    # shapes whose LDS fits four wavefronts per workgroup but not eight at d = 128
    (128, 3, 3, 16, 4, 1, 1), (128, 3, 3, 32, 8, 1, 1), (128, 4, 4, 16, 2, 2, 1), (128, 4, 2, 32, 8, 2, 1),
    (128, 2.5, 3, 32, 16, 2, 1), (128, 3, 4, 16, 1, 1, 3)])
def test_decode_vq_matrix_core_row_groups(d, bits, v_bits, group, n_qh, n_kv, n_q):
    run_decode_vq_case(d, bits, v_bits, group, 2, n_qh, n_kv, n_q, [300, 129], seed=int(1400 + d + 10 * bits + v_bits),
                       want_scores=False)


def test_decode_vq_long_sequence_many_items_and_errors():
    run_decode_vq_case(128, 3, 3, 32, 2, 4, 1, 1, [9000, 3000], seed=1301, want_scores=False)
    cb = binding.octopus_build_codebooks(128, 3)
    q = torch.zeros((1, 1, 4, 128), dtype=torch.float32, device=DEV)
    out = torch.zeros_like(q)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 4, 1, 1, 64), dtype=torch.uint8, device=DEV)
    cache = torch.zeros(binding.octopus_cache_bytes(cb, 1, 1, 64), dtype=torch.uint8, device=DEV)
    vq = torch.zeros(binding.octopus_vq_bytes(128, 3, 32, 1, 1, 64), dtype=torch.uint8, device=DEV)
    sg = torch.zeros((1, 16), dtype=torch.uint8, device=DEV)
    lens = torch.tensor([64], dtype=torch.int32, device=DEV)
    for bad_bits, bad_group in ((5, 32), (3, 8), (0, 32)):
        with pytest.raises(binding.OctopusError):
            binding.octopus_attn_decode_vq(cb, q, sg, cache, 64, vq, bad_bits, bad_group, 1, lens, 64, 1.0, out, ws)
    assert binding.octopus_vq_row_bytes(128, 5, 32) == 0 and binding.octopus_vq_row_bytes(100, 3, 32) == 0
