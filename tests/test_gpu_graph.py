"""The decode and encode calls inside a captured HIP graph: the library allocates nothing, synchronises nothing and
launches on the caller's stream, so a serving loop can capture a step once and replay it.  Every replay is checked
against the eager call on the same inputs (bit for bit: same kernels, same launch shapes), with eager work and
synchronisations between the replays and the inputs changed in place."""
import numpy as np
import pytest

from paper_2605_21226_amd import binding, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, sign_bits_dev, to_dev  # noqa: E402
from test_gpu_parity import make_inputs  # noqa: E402


def test_append_and_decode_step_replayed_from_a_graph():
    d, bits, n_seq, n_kv, g, cap = 128, 3, 3, 2, 4, 512
    cb = binding.octopus_build_codebooks(d, bits)
    keys, vals, signs = make_inputs(4242, n_seq, n_kv, cap, d, "bf16")          # keys [n_seq, cap, n_kv, d]
    k_dev, v_dev, s_dev = to_dev(keys, "bf16"), to_dev(vals, "bf16"), sign_bits_dev(signs)
    n_qh = n_kv * g
    start = [300, 17, 450]

    def fresh_state():
        cache = torch.zeros(binding.octopus_cache_bytes(cb, n_seq, n_kv, cap), dtype=torch.uint8, device=DEV)
        for s, n in enumerate(start):                                            # prefill, eager
            binding.octopus_encode(cb, k_dev[s:s + 1, :n], s_dev, cache[s * (cache.numel() // n_seq):(s + 1) * (cache.numel() // n_seq)], cap)
        return cache

    # static buffers of the step: one new key per sequence, its position, the lengths, the query, the output
    new_key = torch.zeros((n_seq, 1, n_kv, d), dtype=torch.bfloat16, device=DEV)
    pos = torch.zeros(n_seq, dtype=torch.int32, device=DEV)
    lens = torch.zeros(n_seq, dtype=torch.int32, device=DEV)
    q = torch.zeros((n_seq, 1, n_qh, d), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((n_seq, 1, n_qh, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, 1, cap), dtype=torch.uint8, device=DEV)
    scale = 1.0 / np.sqrt(d)

    def step(cache):       # append the new token of every sequence, then attend over the cache including it
        binding.octopus_encode(cb, new_key, s_dev, cache, cap, pos)
        binding.octopus_attn_decode(cb, q, s_dev, cache, cap, v_dev, lens, cap, scale, out, ws)

    def set_inputs(t):     # decode step t: positions start[s] + t
        for s in range(n_seq):
            new_key[s, 0] = k_dev[s, start[s] + t]
        pos.copy_(torch.tensor([n + t for n in start], dtype=torch.int32))
        lens.copy_(torch.tensor([n + t + 1 for n in start], dtype=torch.int32))
        q_t = np.random.default_rng(100 + t).standard_normal((n_seq, 1, n_qh, d)).astype(np.float32)
        q.copy_(to_dev(synth.round_to_bf16(q_t), "bf16"))

    # eager reference: five steps on a cache of its own
    cache_e = fresh_state()
    want = []
    for t in range(5):
        set_inputs(t)
        step(cache_e)
        torch.cuda.synchronize()
        want.append(out.clone())
    assert all(bool(torch.isfinite(w).all()) for w in want) and not torch.equal(want[0], want[1])

    # the same five steps, the step captured once (the eager steps above have loaded every kernel) and replayed
    cache_g = fresh_state()
    set_inputs(0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cache_g)
    for t in range(5):
        set_inputs(t)                                  # eager work between the replays
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want[t]), t
    assert torch.equal(cache_g, cache_e)
