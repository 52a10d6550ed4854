"""GPU parity at the full sizes of the named workloads, in the launch configuration bench.py times:
the whole batch is generated in device memory, encoded and attended by the HIP path in one call each,
and sampled (sequence, KV head) pairs are read back and checked against the CPU oracle — every key
of a sampled pair for the packed codes, every query head of the pair's group for the output."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, layout, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, check_out  # noqa: E402
from paper_2605_21226_amd.synth_device import device_inputs  # noqa: E402


def region_records(cb, cache, n_kv, cap, s, h, n_tok):
    """canonical records [n_tok, record_bytes] and padding of one (sequence, KV head) region"""
    nbytes = cap * cb.plan.granules * 16
    reg = cache[(s * n_kv + h) * nbytes:(s * n_kv + h + 1) * nbytes].cpu().numpy()
    rec, pad = layout.cache_to_records(reg, 1, 1, cap, cb.plan.granules, cb.plan.record_bytes, n_tokens=n_tok)
    return rec[0, 0], pad[0, 0]


def check_pair_codes(plan, k, signs_h, got, tag):
    ref = oracle.encode(plan, k, signs_h)
    g_got = got[:, :4].copy().view(np.float32)[:, 0].astype(np.float64)
    g_ref = ref[:, :4].copy().view(np.float32)[:, 0].astype(np.float64)
    assert np.all(np.abs(g_got - g_ref) <= 1e-6 * np.maximum(g_ref, 1e-30)), tag
    n = k.shape[0] * plan.n_tri
    if np.array_equal(got[:, 4:], ref[:, 4:]):
        return np.array([n, 0, 0], dtype=np.int64)
    return np.array(oracle.classify(plan, k, signs_h, got, tol=1e-6), dtype=np.int64)


def run_full_size(name, bits, pairs, q_rows, seed=0, chunked_encode=False):
    """pairs: (sequence, KV head) pairs to check; q_rows: query positions (of n_q) to check"""
    base = synth.WORKLOADS[name]
    wl = synth.Workload(**{**base.__dict__, "bits": bits})
    cb = binding.octopus_build_codebooks(wl.head_dim, bits)
    plan = oracle.make_plan(wl.head_dim, bits)
    print(f"[full] {name} b={bits}: generating inputs", flush=True)
    keys, vals, q, signs, lens = device_inputs(wl, seed, DEV)
    cap, n_kv, d = wl.n_tokens, wl.n_kv_heads, wl.head_dim
    cap = -(-cap // 64) * 64
    if cap != wl.n_tokens:        # values need t_capacity rows
        v2 = torch.zeros((wl.n_seq, n_kv, cap, d), dtype=vals.dtype, device=DEV)
        v2[:, :, :wl.n_tokens] = vals
        vals = v2
    sbits = torch.from_numpy(synth.sign_bits(signs)).to(DEV)
    cache = torch.zeros(binding.octopus_cache_bytes(cb, wl.n_seq, n_kv, cap), dtype=torch.uint8, device=DEV)
    print(f"[full] {name} b={bits}: encode", flush=True)
    if chunked_encode:            # bulk prefill, then the workload's chunk appended at its position
        n0 = wl.n_tokens - wl.n_new
        binding.octopus_encode(cb, keys[:, :n0], sbits, cache, cap)
        sp = torch.full((wl.n_seq,), n0, dtype=torch.int32, device=DEV)
        binding.octopus_encode(cb, keys[:, n0:], sbits, cache, cap, sp)
    else:
        binding.octopus_encode(cb, keys, sbits, cache, cap)
    torch.cuda.synchronize()
    max_len = int(lens.max())
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, wl.n_seq, wl.n_q_heads, n_kv, wl.n_q, max_len),
                     dtype=torch.uint8, device=DEV)
    out = torch.full((wl.n_seq, wl.n_q, wl.n_q_heads, d), float("nan"), dtype=torch.float32, device=DEV)
    scale = 1.0 / float(np.sqrt(d))
    print(f"[full] {name} b={bits}: decode attention", flush=True)
    binding.octopus_attn_decode(cb, q, sbits, cache, cap, vals, torch.from_numpy(lens).to(DEV), max_len, scale, out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())

    g = wl.n_q_heads // n_kv
    total = np.zeros(3, dtype=np.int64)
    worst = 0.0
    for (s, h) in pairs:
        print(f"[full] {name} b={bits}: oracle on sequence {s}, KV head {h}", flush=True)
        L = int(lens[s])
        k = keys[s, :, h].float().cpu().numpy().astype(np.float64)             # every cached token of the pair
        rec, pad = region_records(cb, cache, n_kv, cap, s, h, wl.n_tokens)
        assert not pad.any()
        total += check_pair_codes(plan, k, signs[h], rec, f"{name} b={bits} ({s},{h})")
        v = vals[s, h, :L].float().cpu().numpy().astype(np.float64)
        qq = q[s][q_rows][:, h * g:(h + 1) * g].float().cpu().numpy().astype(np.float64).reshape(-1, d)
        _, ref, gap = oracle.attention(plan, rec[:L], signs[h], qq, v, scale)    # the codes the GPU wrote
        assert gap < 1e-9
        got = out[s][q_rows][:, h * g:(h + 1) * g].cpu().numpy().reshape(-1, d)
        for r in range(ref.shape[0]):
            worst = max(worst, check_out(got[r], ref[r]))
    print(f"[full] {name} b={bits}: triplets equal={total[0]} boundary_ties={total[1]} hard={total[2]}; "
          f"worst output error {worst:.3g} (relative to the row's max)", flush=True)
    assert total[2] == 0
    assert total[1] <= max(2, 2e-4 * total.sum())
    del keys, vals, cache, out, ws
    torch.cuda.empty_cache()


def test_full_llama3_8b_decode():
    run_full_size("llama3_8b_decode", 3.0, [(0, 0), (7, 3), (15, 7), (9, 5)], [0])


def test_full_long_context_2bit():
    run_full_size("long_context_2bit", 2.0, [(0, 1), (3, 6)], [0])


def test_full_causal_video_chunk():
    run_full_size("causal_video", 4.0, [(0, 0), (0, 13), (0, 23)], [0, 1, 1799, 3598, 3599], chunked_encode=True)


@pytest.mark.parametrize("bits", [1.5, 2, 2.5, 3, 4])
def test_full_ragged_d256(bits):
    lens = synth.context_lengths(0, synth.WORKLOADS["ragged_d256"])
    s_short, s_long = int(np.argmin(lens)), int(np.argmax(lens))
    run_full_size("ragged_d256", float(bits), [(s_short, 0), (s_long, 7)], [0])
