"""GPU parity of the optional 1-bit QJL residual (Sec. 3.6): the side-car written by octopus_encode_qjl
against the oracle's, computed from the codes the GPU itself wrote (so that a tie in the codes does not
masquerade as a side-car error).  Sign bits must match except where the oracle's rotated residual
coordinate is within 1e-6 of zero (counted); gamma_r within one fp16 unit in the last place."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, layout, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, new_cache, sign_bits_dev, to_dev  # noqa: E402
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
    n_flip = n_total = 0
    for s in range(n_seq):
        for h in range(n_kv):
            k = keys[s, :n_tok, h].astype(np.float64)
            sigma, g_ref = oracle.qjl_encode(plan, k, signs[h], signs2[h], rec[s, h, :n_tok])
            got = np.unpackbits(bits[s, h, :n_tok], axis=-1, bitorder="little")       # 1 = negative
            want = (sigma < 0).astype(np.uint8)
            g_got = gamma_r[s, h, :n_tok].astype(np.float64)
            ulp = np.maximum(np.spacing(np.float16(g_ref).astype(np.float16)).astype(np.float64), 2.0 ** -24)
            assert np.all(np.abs(g_got - g_ref) <= ulp), f"{tag}: gamma_r off by more than one fp16 ulp"
            n_total += want.size
            for t, j in zip(*np.nonzero(got != want)):
                e_dir, e_nrm = oracle.unpack_record(plan, rec[s, h, t])[1:]
                _, _, r = oracle.qjl_residual(plan, k[t], signs[h], signs2[h], e_dir, e_nrm)
                y = oracle.rotate(r, signs2[h])
                assert abs(y[j]) <= 1e-6, f"{tag}: sign bit ({s},{h},{t},{j}) differs where |y| = {abs(y[j]):.3g}"
                n_flip += 1
    print(f"[qjl] {tag}: {n_total} sign bits, {n_flip} differ at |y| <= 1e-6")
    assert n_flip <= max(2, 1e-4 * n_total)


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
