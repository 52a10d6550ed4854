"""GPU parity of the encoder's rounding variants (App. E): octopus_encode_rounding against the oracle in
the same mode; codes bit-exact, decision-boundary ties within 1e-6 counted, as for the default encoder."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, layout

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, gpu_encode, new_cache, sign_bits_dev, to_dev  # noqa: E402
from test_gpu_parity import compare_records, make_inputs  # noqa: E402

# binding constant -> the oracle's mode
MODES = {binding.ROUND_SEED: oracle.MODE_SCALAR, binding.ROUND_LOCAL_3X3: oracle.MODE_LOCAL_3X3,
         binding.ROUND_FULL: oracle.MODE_FULL, binding.ROUND_INDEPENDENT: oracle.MODE_INDEPENDENT,
         binding.ROUND_LOCAL_2X2: oracle.MODE_LOCAL_2X2}


def gpu_encode_rounding(cb, keys, dtype, signs, cap, rounding, start_pos=None, cache=None):
    n_seq, _, n_kv, _ = keys.shape
    if cache is None:
        cache = new_cache(cb, n_seq, n_kv, cap)
    sp = None if start_pos is None else torch.tensor(start_pos, dtype=torch.int32, device=DEV)
    binding.octopus_encode_rounding(cb, to_dev(keys, dtype), sign_bits_dev(signs), cache, cap, rounding, sp)
    torch.cuda.synchronize()
    rec, pad = layout.cache_to_records(cache.cpu().numpy(), n_seq, n_kv, cap, cb.plan.granules, cb.plan.record_bytes)
    return rec, pad


@pytest.mark.parametrize("rounding", sorted(MODES))
@pytest.mark.parametrize("d,bits", [(64, 2), (64, 4), (128, 1), (128, 1.5), (128, 3), (128, 4), (256, 2.5), (256, 3)])
def test_encode_rounding_modes(d, bits, rounding):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, _, signs = make_inputs(int(1000 + d + 10 * bits + rounding), 2, 2, 200, d, "bf16")   # 3 tiles + a tail of 8
    rec, pad = gpu_encode_rounding(cb, keys, "bf16", signs, 256, rounding)
    assert not pad.any() and not rec[:, :, 200:].any()
    compare_records(plan, keys, signs, rec, f"d={d} b={bits} rounding={rounding}", mode=MODES[rounding])


def test_rounding_3x3_is_the_default_encoder_and_modes_differ():
    d = 128
    cb = binding.octopus_build_codebooks(d, 3)
    keys, _, signs = make_inputs(55, 1, 2, 300, d, "fp32")
    recs = {r: gpu_encode_rounding(cb, keys, "fp32", signs, 320, r)[0] for r in MODES}
    plain, _, _ = gpu_encode(cb, keys, "fp32", signs, 320)
    assert np.array_equal(recs[binding.ROUND_LOCAL_3X3], plain)
    assert np.array_equal(recs[binding.ROUND_FULL], plain)            # Sec. 3.5: 3x3 reaches the full-grid optimum here
    for r in (binding.ROUND_SEED, binding.ROUND_INDEPENDENT, binding.ROUND_LOCAL_2X2):
        assert not np.array_equal(recs[r], plain)


def test_rounding_append_and_bad_mode():
    d = 64
    cb = binding.octopus_build_codebooks(d, 3)
    plan = oracle.make_plan(d, 3)
    keys, _, signs = make_inputs(56, 2, 1, 70, d, "bf16")
    start = [3, 100]
    cache = new_cache(cb, 2, 1, 192, fill=0xCD)
    rec, _ = gpu_encode_rounding(cb, keys, "bf16", signs, 192, binding.ROUND_LOCAL_2X2, start_pos=start, cache=cache)
    for s, st in enumerate(start):
        assert np.all(rec[s, :, :st] == 0xCD) and np.all(rec[s, :, st + 70:] == 0xCD)
        compare_records(plan, keys[s:s + 1], signs, rec[s:s + 1, :, st:st + 70], f"append at {st}",
                        mode=oracle.MODE_LOCAL_2X2)
    with pytest.raises(binding.OctopusError):
        gpu_encode_rounding(cb, keys, "bf16", signs, 192, 7)
