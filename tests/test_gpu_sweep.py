"""The bit-allocation sweep of App. D on the GPU: for each of the 13 printed (b_dir, b_nrm) pairs at d = 128 the HIP
encoder's codes are (a) the oracle's, bit for bit up to counted 1e-6 ties, and (b) decoded by the oracle they
reproduce the printed MSE and 1 - cos (n = 8192 keys, 4 rotation seeds); the split-K decode kernel of every pair is
checked against the oracle's attention on a small ragged batch."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from conftest import read_golden  # noqa: E402
from gpu_util import cache_from_records, check_out, gpu_decode, gpu_encode  # noqa: E402
from test_gpu_parity import compare_records, make_inputs, oracle_attention_all  # noqa: E402

D = 128
PAIRS = [(int(r[0]), int(r[1]), float(r[2]), float(r[3])) for r in read_golden("bit_split_diagonal.txt")]


def _close(got, printed, rel, digits):
    return abs(got - printed) <= rel * abs(printed) + 0.5 * 10.0 ** (-digits)


@pytest.mark.parametrize("b_dir,b_nrm,mse,omc", PAIRS)
def test_sweep_pair_codes_and_printed_statistics(b_dir, b_nrm, mse, omc):
    cb = binding.octopus_build_codebooks_pair(D, b_dir, b_nrm)
    plan = oracle.make_plan_pair(D, b_dir, b_nrm)
    got_mse, got_cos = [], []
    for seed in range(4):
        keys = synth.gaussian_keys(seed, 8192, D)                       # the keys of the oracle's own table test
        s = synth.sign_vectors(seed, 1, D)
        rec, pad, _ = gpu_encode(cb, keys[None, :, None, :], "fp32", s, 8192)
        assert not pad.any()
        compare_records(plan, keys[None, :, None, :].astype(np.float32), s, rec, f"pair ({b_dir},{b_nrm}) seed {seed}")
        k_hat = oracle.reconstruct(plan, rec[0, 0], s[0])              # the GPU's codes, decoded by the oracle
        k32 = keys.astype(np.float32).astype(np.float64)
        got_mse.append(np.mean((k_hat - k32) ** 2))
        got_cos.append(np.mean(np.sum(k_hat * k32, axis=1) / (np.linalg.norm(k_hat, axis=1) * np.linalg.norm(k32, axis=1))))
    m, c = float(np.mean(got_mse)), float(np.mean(got_cos))
    print(f"[sweep] ({b_dir},{b_nrm}): MSE {m:.4f} (printed {mse}), 1-cos {1 - c:.4f} (printed {omc})")
    assert _close(m, mse, 0.015, 4) and _close(1 - c, omc, 0.015, 4)


@pytest.mark.parametrize("b_dir,b_nrm", [(p[0], p[1]) for p in PAIRS])
def test_sweep_pair_decode_attention(b_dir, b_nrm):
    cb = binding.octopus_build_codebooks_pair(D, b_dir, b_nrm)
    plan = oracle.make_plan_pair(D, b_dir, b_nrm)
    n_seq, n_kv, g, lens = 3, 2, 4, [333, 64, 700]
    T = max(lens)
    cap = -(-T // 64) * 64
    keys, vals, signs = make_inputs(500 + 10 * b_dir + b_nrm, n_seq, n_kv, T, D, "bf16")
    rec = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                    for s in range(n_seq)])
    q = synth.queries(7, synth.Workload("t", n_seq, n_kv * g, n_kv, D, T, 3.0, "bf16"))
    v = np.zeros((n_seq, n_kv, cap, D), dtype=np.float32)
    v[:, :, :T] = vals
    scale = 1.0 / np.sqrt(D)
    out, _ = gpu_decode(cb, q, "bf16", signs, cache_from_records(cb, rec, cap), cap, v, "bf16", lens, scale, want_scores=False)
    ref, _ = oracle_attention_all(plan, rec, signs, q.astype(np.float64), v.astype(np.float64), lens, scale)
    for s in range(n_seq):
        for h in range(n_kv * g):
            check_out(out[s, 0, h], ref[s, 0, h])


def test_sweep_only_pairs_refuse_the_variants():
    cb = binding.octopus_build_codebooks_pair(D, 3, 3)
    keys = torch.zeros((1, 64, 1, D), dtype=torch.bfloat16, device="cuda:0")
    signs = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    cache = torch.zeros(binding.octopus_cache_bytes(cb, 1, 1, 64), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_encode_rounding(cb, keys, signs, cache, 64, binding.ROUND_FULL)
    assert err.value.code == binding.EUNSUPPORTED
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 1, 1, 1, 64), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros((1, 1, 1, D), dtype=torch.float32, device="cuda:0")
    lens = torch.tensor([64], dtype=torch.int32, device="cuda:0")
    v32 = torch.zeros((1, 1, 64, D), dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.OctopusError) as err:     # fp32 values: the vector-unit kernel is not built for these pairs
        binding.octopus_attn_decode(cb, keys[:, :1], signs, cache, 64, v32, lens, 64, 0.1, out, ws)
    assert err.value.code == binding.EUNSUPPORTED
