"""The entry point that allocates nothing (octopus_attn_decode_static: the library's static scratch array in place of
a caller workspace), through the C ABI, against octopus_attn_decode on the same inputs: two calls in a row, the second
with a smaller input, and the refusal of shapes beyond the array."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, check_out, check_scores, cache_from_records, sign_bits_dev, to_dev  # noqa: E402
from test_gpu_parity import make_inputs, oracle_attention_all  # noqa: E402


def run_case(seed, n_seq, n_kv, g, n_tok, lens, d=128, bits=3, dtype="bf16"):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    cap = -(-n_tok // 64) * 64
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, n_tok, d, dtype)
    rec = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                    for s in range(n_seq)])
    cache = cache_from_records(cb, rec, cap)
    v = np.zeros((n_seq, n_kv, cap, d), dtype=np.float32)
    v[:, :, :n_tok] = vals
    rng = np.random.default_rng(seed + 77)
    q = rng.standard_normal((n_seq, 1, n_kv * g, d)).astype(np.float32)
    if dtype == "bf16":
        q = synth.round_to_bf16(q)
    scale = 1.0 / np.sqrt(d)
    q_dev, v_dev, s_dev = to_dev(q, dtype), to_dev(v, dtype), sign_bits_dev(signs)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    max_len = int(max(lens))
    outs, scores = [], []
    for static in (False, True):
        out = torch.full((n_seq, 1, n_kv * g, d), float("nan"), dtype=torch.float32, device=DEV)
        sc = torch.full((n_seq, 1, n_kv * g, cap), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            binding.octopus_attn_decode_static(cb, q_dev, s_dev, cache, cap, v_dev, lens_dev, max_len, scale, out, sc)
        else:
            ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_kv * g, n_kv, 1, max_len),
                             dtype=torch.uint8, device=DEV)
            binding.octopus_attn_decode(cb, q_dev, s_dev, cache, cap, v_dev, lens_dev, max_len, scale, out, ws, sc)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        scores.append(sc.cpu().numpy())
    # same kernels, same launch shapes: the two entry points agree bit for bit ...
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(np.nan_to_num(scores[0], nan=-1.0), np.nan_to_num(scores[1], nan=-1.0))
    # ... and with the oracle to the bar of every other decode test
    ref_out, ref_scores = oracle_attention_all(plan, rec, signs, q.astype(np.float64), v.astype(np.float64), lens, scale)
    for s in range(n_seq):
        L = int(lens[s])
        for h in range(n_kv * g):
            check_out(outs[1][s, 0, h], ref_out[s, 0, h])
            check_scores(scores[1][s, 0, h, :L], ref_scores[(s, h // g)][0, h % g])


def test_static_scratch_matches_workspace_entry_point_twice_second_call_smaller():
    run_case(21, 3, 2, 4, 700, [700, 333, 64])
    run_case(22, 1, 1, 4, 150, [150])


def test_static_scratch_refuses_shapes_beyond_the_array():
    cb = binding.octopus_build_codebooks(64, 4)
    # 24 heads x 3600 query rows against 75,600 tokens: the partials of the many-row kernel exceed 32 MiB
    need = binding.octopus_attn_decode_workspace(cb, 1, 24, 24, 3600, 75648)
    assert need > binding.STATIC_SCRATCH_BYTES
    q = torch.zeros((1, 3600, 24, 64), dtype=torch.bfloat16, device=DEV)
    v = torch.zeros((1, 24, 75648, 64), dtype=torch.bfloat16, device=DEV)
    cache = torch.zeros(binding.octopus_cache_bytes(cb, 1, 24, 75648), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 3600, 24, 64), dtype=torch.float32, device=DEV)
    lens = torch.tensor([75600], dtype=torch.int32, device=DEV)
    signs = torch.zeros(24 * 8, dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_attn_decode_static(cb, q, signs, cache, 75648, v, lens, 75600, 0.125, out)
    assert err.value.code == binding.ESCRATCH
