"""GPU parity of the optional 1-bit QJL residual (Sec. 3.6).

Encoder: the side-car written by octopus_encode_qjl against the oracle's, on the keys whose GPU record equals
the oracle's record (a key whose codes differ by a rounding tie has another residual; such keys are counted
and are covered by the record comparison of the plain encoder).  Sign bits must match except where the
oracle's rotated residual coordinate is within 1e-6 of zero (counted); gamma_r within one fp16 unit in the
last place.

Decoder: octopus_attn_decode_qjl over the oracle's records and side-car, brought into the device layouts,
against the oracle's corrected attention: scores and outputs to the 1e-3 bar of the plain decoder."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, layout, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import (DEV, cache_from_records, check_out, check_scores, new_cache, record_gammas, score_floor,  # noqa: E402
                      sign_bits_dev, to_dev)
from test_gpu_parity import make_inputs  # noqa: E402


def gpu_encode_qjl(cb, keys, dtype, signs, signs2, cap, start_pos=None):
    n_seq, n_new, n_kv, d = keys.shape
    cache = new_cache(cb, n_seq, n_kv, cap)
    qjl = torch.zeros(binding.octopus_qjl_bytes(cb, n_seq, n_kv, cap), dtype=torch.uint8, device=DEV)
    sp = None if start_pos is None else torch.tensor(start_pos, dtype=torch.int32, device=DEV)
    binding.octopus_encode_qjl(cb, to_dev(keys, dtype), sign_bits_dev(signs), sign_bits_dev(signs2), cache, qjl, cap, sp)
    torch.cuda.synchronize()
    rec, _ = layout.cache_to_records(cache.cpu().numpy(), n_seq, n_kv, cap, cb.plan.granules, cb.plan.record_bytes)
    bits, gamma_r = layout.qjl_to_canonical(qjl.cpu().numpy(), n_seq, n_kv, cap, d)
    return rec, bits, gamma_r, cache, qjl


def check_sidecar(plan, keys, signs, signs2, rec, bits, gamma_r, n_tok, tag):
    n_seq, _, n_kv, d = keys.shape
    n_flip = n_total = n_other = 0
    for s in range(n_seq):
        for h in range(n_kv):
            k = keys[s, :n_tok, h].astype(np.float64)
            ref_rec = oracle.encode(plan, k, signs[h])
            same = np.all(ref_rec[:, 4:] == rec[s, h, :n_tok, 4:], axis=1)      # codes equal (gamma: fp32 norm)
            n_other += int(np.sum(~same))
            sigma, g_ref = oracle.qjl_encode(plan, k, signs[h], signs2[h], ref_rec)
            got = np.unpackbits(bits[s, h, :n_tok], axis=-1, bitorder="little")       # 1 = negative
            want = (sigma < 0).astype(np.uint8)
            g_got = gamma_r[s, h, :n_tok].astype(np.float64)
            ulp = np.maximum(np.spacing(np.float16(g_ref).astype(np.float16)).astype(np.float64), 2.0 ** -24)
            assert np.all((np.abs(g_got - g_ref) <= ulp)[same]), f"{tag}: gamma_r off by more than one fp16 ulp"
            n_total += int(np.sum(same)) * d
            for t, j in zip(*np.nonzero((got != want) & same[:, None])):
                e_dir, e_nrm = oracle.unpack_record(plan, ref_rec[t])[1:]
                _, _, r = oracle.qjl_residual(plan, k[t], signs[h], signs2[h], e_dir, e_nrm)
                y = oracle.rotate(r, signs2[h])
                assert abs(y[j]) <= 1e-6, f"{tag}: sign bit ({s},{h},{t},{j}) differs where |y| = {abs(y[j]):.3g}"
                n_flip += 1
    print(f"[qjl] {tag}: {n_total} sign bits, {n_flip} differ at |y| <= 1e-6; {n_other} keys with other codes skipped")
    assert n_flip <= max(2, 1e-4 * n_total)
    assert n_other <= max(2, 2e-3 * n_seq * n_kv * n_tok)


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("bits", [1.5, 2, 3, 4])
def test_encode_qjl_sidecar(d, bits):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, _, signs = make_inputs(int(500 + d + 10 * bits), 2, 2, 200, d, "bf16")
    signs2 = synth.sign_vectors(int(900 + d), 2, d)
    rec, sbits, gamma_r, _, _ = gpu_encode_qjl(cb, keys, "bf16", signs, signs2, 256)
    # the records are those of the plain encoder
    from gpu_util import gpu_encode
    rec_plain, _, _ = gpu_encode(cb, keys, "bf16", signs, 256)
    assert np.array_equal(rec, rec_plain)
    assert not sbits[:, :, 200:].any() and not gamma_r[:, :, 200:].any()          # untouched slots stay zero
    check_sidecar(plan, keys, signs, signs2, rec, sbits, gamma_r, 200, f"d={d} b={bits}")


def test_encode_qjl_append_and_fp32_keys():
    d = 128
    cb = binding.octopus_build_codebooks(d, 3)
    plan = oracle.make_plan(d, 3)
    keys, _, signs = make_inputs(77, 2, 1, 90, d, "fp32")
    signs2 = synth.sign_vectors(78, 1, d)
    start = [5, 130]
    rec, sbits, gamma_r, _, _ = gpu_encode_qjl(cb, keys, "fp32", signs, signs2, 256, start_pos=start)
    for s, st in enumerate(start):
        assert not sbits[s, :, :st].any() and not sbits[s, :, st + 90:].any()
        check_sidecar(plan, keys[s:s + 1], signs, signs2, rec[s:s + 1, :, st:st + 90], sbits[s:s + 1, :, st:st + 90],
                      gamma_r[s:s + 1, :, st:st + 90], 90, f"append at {st}")


# ---- decode attention with the corrected score ---------------------------------------------------------

def run_decode_qjl_case(d, bits, n_seq, n_qh, n_kv, n_q, lens, seed, t_capacity=None, want_scores=True):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    T = max(int(max(lens)), 1)
    t_capacity = t_capacity or -(-T // 64) * 64
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")
    signs2 = synth.sign_vectors(seed + 1000, n_kv, d)
    records = np.zeros((n_seq, n_kv, T, plan.record_bytes), dtype=np.uint8)
    sigma = np.zeros((n_seq, n_kv, T, d), dtype=np.int8)
    gamma_r = np.zeros((n_seq, n_kv, T), dtype=np.float64)
    for s in range(n_seq):
        for h in range(n_kv):
            k = keys[s, :, h].astype(np.float64)
            records[s, h] = oracle.encode(plan, k, signs[h])
            sigma[s, h], gamma_r[s, h] = oracle.qjl_encode(plan, k, signs[h], signs2[h], records[s, h])
    assert np.array_equal(gamma_r, gamma_r.astype(np.float16).astype(np.float64))     # already fp16 values
    wl = synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16", n_q=n_q)
    q = synth.queries(seed, wl)
    v = np.zeros((n_seq, n_kv, t_capacity, d), dtype=np.float32)
    v[:, :, :T] = vals
    scale = 1.0 / np.sqrt(d)
    # the oracle's codes and side-car in the device layouts
    cache = cache_from_records(cb, records, t_capacity)
    sbits = np.packbits((sigma < 0).astype(np.uint8), axis=-1, bitorder="little")
    qjl = torch.from_numpy(layout.qjl_from_canonical(sbits, gamma_r.astype(np.float16), t_capacity)).to(DEV)
    assert qjl.numel() == binding.octopus_qjl_bytes(cb, n_seq, n_kv, t_capacity)

    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, T), dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    scores = (torch.full((n_seq, n_q, n_qh, t_capacity), float("nan"), dtype=torch.float32, device=DEV)
              if want_scores else None)
    lens_dev = torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV)
    binding.octopus_attn_decode_qjl(cb, to_dev(q, "bf16"), sign_bits_dev(signs), sign_bits_dev(signs2), cache, qjl,
                                    t_capacity, to_dev(v, "bf16"), lens_dev, T, scale, out, ws, scores)
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
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            ref_s, ref_o = oracle.attention_qjl(plan, records[s, h, :L], signs[h], signs2[h], sigma[s, h, :L],
                                                gamma_r[s, h, :L], qq, v[s, h, :L].astype(np.float64), scale)
            ref_s, ref_o = ref_s.reshape(n_q, g, L), ref_o.reshape(n_q, g, d)
            plain_s, _, _ = oracle.attention(plan, records[s, h, :L], signs[h], qq, v[s, h, :L].astype(np.float64), scale)
            assert np.max(np.abs(plain_s.reshape(n_q, g, L) - ref_s)) > 1e-3     # the correction is visible at this bar
            for qi in range(n_q):
                for j in range(g):
                    if want_scores:
                        floor = score_floor(q[s, qi, h * g + j], record_gammas(records[s, h, :L]), scale)
                        worst_s = max(worst_s, check_scores(scores[s, qi, h * g + j, :L], ref_s[qi, j], floor))
                    worst_o = max(worst_o, check_out(out[s, qi, h * g + j], ref_o[qi, j]))
        if want_scores:
            assert np.all(np.isnan(scores[s, :, :, L:]))
    print(f"[attn-qjl] d={d} b={bits} lens={list(lens)}: worst score err {worst_s:.3g} x tol, worst out err {worst_o:.3g}")


@pytest.mark.parametrize("bits", [1, 1.5, 2, 2.5, 3, 4])
def test_decode_qjl_gqa_ragged_d128(bits):
    run_decode_qjl_case(128, bits, 3, 8, 2, 1, [0, 77, 1000], seed=int(600 + 10 * bits))


@pytest.mark.parametrize("bits", [2, 3])
def test_decode_qjl_d64_multi_query(bits):
    run_decode_qjl_case(64, bits, 1, 3, 3, 5, [700], seed=int(700 + 10 * bits))


@pytest.mark.parametrize("bits", [2, 4])
def test_decode_qjl_d256(bits):
    run_decode_qjl_case(256, bits, 2, 4, 2, 1, [513, 64], seed=int(800 + 10 * bits))


def test_decode_qjl_several_row_groups_and_long_sequence():
    run_decode_qjl_case(128, 3, 1, 6, 1, 1, [300], seed=901)                        # 6 rows -> groups of 4
    run_decode_qjl_case(256, 3, 1, 3, 1, 1, [200], seed=902)                        # 3 rows -> groups of 2
    run_decode_qjl_case(128, 2, 2, 4, 1, 1, [9000, 3000], seed=903, want_scores=False)   # many work items


def test_decode_qjl_argument_errors():
    cb = binding.octopus_build_codebooks(128, 3)
    q = torch.zeros((1, 1, 4, 128), dtype=torch.float32, device=DEV)
    v32 = torch.zeros((1, 1, 64, 128), dtype=torch.float32, device=DEV)
    out = torch.zeros((1, 1, 4, 128), dtype=torch.float32, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 4, 1, 1, 64), dtype=torch.uint8, device=DEV)
    cache = new_cache(cb, 1, 1, 64)
    qjl = torch.zeros(binding.octopus_qjl_bytes(cb, 1, 1, 64), dtype=torch.uint8, device=DEV)
    sg = torch.zeros((1, 16), dtype=torch.uint8, device=DEV)
    lens = torch.tensor([64], dtype=torch.int32, device=DEV)
    with pytest.raises(binding.OctopusError):        # fp32 values are not served with the residual
        binding.octopus_attn_decode_qjl(cb, q, sg, sg, cache, qjl, 64, v32, lens, 64, 1.0, out, ws)
    with pytest.raises(binding.OctopusError):        # side-car missing
        binding.octopus_attn_decode_qjl(cb, q, sg, sg, cache, None, 64, v32.to(torch.bfloat16), lens, 64, 1.0, out, ws)
