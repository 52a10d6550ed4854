"""GPU parity on seeded random shapes: head dimension, bit width, GQA ratio, query count, batch size and
ragged lengths (empty sequences, single tokens, one long sequence among short ones) are drawn at random
and every entry point is compared with the oracle through the same case runners as the fixed-shape tests.
The draw is deterministic (fixed seeds), so a failure names a reproducible case."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import test_gpu_hybrid as hybrid  # noqa: E402
import test_gpu_paged as paged  # noqa: E402
import test_gpu_parity as parity  # noqa: E402
import test_gpu_qjl as qjl  # noqa: E402
import test_gpu_values as values  # noqa: E402
from gpu_util import gpu_encode  # noqa: E402


def draw_shape(rng, max_rows=300000, max_tokens=25000):
    """-> d, bits, n_kv, heads per KV head, n_q, lens"""
    while True:
        d = int(rng.choice([64, 128, 256]))
        bits = float(rng.choice(parity.ALL_BITS))
        bits = int(bits) if bits == int(bits) else bits
        n_kv = int(rng.integers(1, 4))
        g = int(rng.choice([1, 2, 3, 4, 5, 8]))
        n_q = int(rng.choice([1, 1, 1, 2, 7, 9, 33, 40]))
        kind = int(rng.integers(0, 3))
        if kind == 0:      # a few sequences of any length
            lens = [int(x) for x in rng.integers(0, 2500, size=int(rng.integers(1, 5)))]
        elif kind == 1:    # many short ones (more work items than workgroups, more sequences than lanes)
            lens = [int(x) for x in rng.integers(0, 300, size=int(rng.integers(5, 90)))]
        else:              # one long sequence among short ones
            lens = [int(x) for x in rng.integers(0, 200, size=int(rng.integers(2, 8)))]
            lens[int(rng.integers(0, len(lens)))] = int(rng.integers(1500, 4000))
        if max(lens) == 0:
            lens[0] = 1
        if sum(lens) * n_kv * g * n_q <= max_rows and sum(lens) * n_kv <= max_tokens:   # bounds the oracle's work
            return d, bits, n_kv, g, n_q, lens


@pytest.mark.parametrize("seed", range(4))
def test_decode_random_shapes(seed):
    rng = np.random.default_rng(9000 + seed)
    for i in range(12):
        d, bits, n_kv, g, n_q, lens = draw_shape(rng)
        dtype = "bf16" if rng.random() < 0.8 else "fp32"
        want_scores = bool(rng.random() < 0.4) and n_q * g <= 16
        cap = -(-max(lens) // 64) * 64 + 64 * int(rng.integers(0, 3))
        print(f"decode seed={seed} case={i}: d={d} bits={bits} n_kv={n_kv} g={g} n_q={n_q} {dtype} "
              f"scores={want_scores} cap={cap} lens={lens}", flush=True)
        parity.run_decode_case(d, bits, len(lens), n_kv * g, n_kv, n_q, lens, dtype, seed=9100 + 100 * seed + i,
                               t_capacity=cap, want_scores=want_scores)


@pytest.mark.parametrize("seed", range(4))
def test_variant_entry_points_random_shapes(seed):
    rng = np.random.default_rng(9500 + seed)
    for i in range(15):
        d, bits, n_kv, g, n_q, lens = draw_shape(rng)
        n_seq = len(lens)
        want_scores = bool(rng.random() < 0.4) and n_q * g <= 16
        case_seed = 9600 + 100 * seed + i
        variant = ("qjl", "vq", "hybrid", "encode", "paged")[i % 5]
        head = f"{variant} seed={seed} case={i}: d={d} bits={bits} n_kv={n_kv} g={g} n_q={n_q} scores={want_scores}"
        if variant == "qjl":
            print(f"{head} lens={lens}", flush=True)
            qjl.run_decode_qjl_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, case_seed, want_scores=want_scores)
        elif variant == "vq":
            v_bits, group = int(rng.choice([2, 3, 4])), int(rng.choice([16, 32]))
            print(f"{head} v_bits={v_bits} group={group} lens={lens}", flush=True)
            values.run_decode_vq_case(d, bits, v_bits, group, n_seq, n_kv * g, n_kv, n_q, lens, case_seed,
                                      want_scores=want_scores)
        elif variant == "paged":
            n_q = min(n_q, 31 // g)          # (chunks of 32 or more query rows per KV head over pages: the test below)
            print(f"{head} lens={lens} n_q={n_q}", flush=True)
            paged.run_paged_decode_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, case_seed,
                                        q_dtype="bf16" if rng.random() < 0.7 else "fp32")
        elif variant == "hybrid":
            w_cap = int(rng.choice([1, 32, 64, 100]))
            win = [int(x) for x in rng.integers(0, w_cap + 1, size=n_seq)]
            dtype = "bf16" if rng.random() < 0.7 else "fp32"
            print(f"{head} {dtype} w_cap={w_cap} win={win} lens={lens}", flush=True)
            hybrid.run_hybrid_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, win, w_cap, dtype, case_seed,
                                   want_scores=want_scores)
        else:
            n_tok, ns = int(rng.integers(1, 700)), int(rng.integers(1, 4))
            dtype = "bf16" if rng.random() < 0.7 else "fp32"
            cap = -(-n_tok // 64) * 64 + 64 * int(rng.integers(0, 2))
            print(f"{head} {dtype} n_seq={ns} n_tok={n_tok} cap={cap}", flush=True)
            cb = binding.octopus_build_codebooks(d, bits)
            plan = oracle.make_plan(d, bits)
            keys, _, signs = parity.make_inputs(case_seed, ns, n_kv, n_tok, d, dtype)
            rec, pad, _ = gpu_encode(cb, keys, dtype, signs, cap)
            assert not pad.any() and not rec[:, :, n_tok:].any()
            parity.compare_records(plan, keys, signs, rec, head)


@pytest.mark.parametrize("seed", range(3))
def test_paged_variant_entry_points_random_shapes(seed):
    """The paged forms of the variants: window, quantised values, QJL side-car, and chunks of many query rows."""
    rng = np.random.default_rng(9800 + seed)
    for i in range(12):
        d, bits, n_kv, g, n_q, lens = draw_shape(rng, max_tokens=12000)
        n_seq = len(lens)
        case_seed = 9900 + 100 * seed + i
        variant = ("hybrid", "vq", "qjl", "many")[i % 4]
        rows = n_q * g
        if variant == "many":
            if d == 256:
                d = 128                                       # (the many-row kernel is built up to d = 128)
            n_q = max(n_q, -(-32 // g))
        elif rows >= 32 and (variant != "hybrid" or d == 256):
            n_q = max(1, 31 // g)                             # those chunks are refused over pages
        head = f"paged {variant} seed={seed} case={i}: d={d} bits={bits} n_kv={n_kv} g={g} n_q={n_q}"
        if variant == "hybrid":
            w_cap = int(rng.choice([1, 32, 64, 100]))
            win = [int(x) for x in rng.integers(0, w_cap + 1, size=n_seq)]
            k_dtype = "bf16" if rng.random() < 0.7 else "fp32"
            print(f"{head} {k_dtype} w_cap={w_cap} win={win} lens={lens}", flush=True)
            paged.run_paged_hybrid_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, win, w_cap, k_dtype, case_seed)
        elif variant == "vq":
            v_bits, group = int(rng.choice([2, 3, 4])), int(rng.choice([16, 32]))
            cb = binding.octopus_build_codebooks(d, bits)
            if not binding.octopus_vq_on_matrix_cores(cb, n_kv * g, n_kv, n_q, v_bits, group):
                v_bits, group, n_q = 3, 32, max(1, min(n_q, 4 // g))     # a shape every plan has a build for
            print(f"{head} v_bits={v_bits} group={group} n_q={n_q} lens={lens}", flush=True)
            assert binding.octopus_vq_on_matrix_cores(cb, n_kv * g, n_kv, n_q, v_bits, group)
            paged.run_paged_vq_decode_case(d, bits, v_bits, group, n_seq, n_kv * g, n_kv, n_q, lens, case_seed)
        elif variant == "qjl":
            print(f"{head} lens={lens}", flush=True)
            paged.run_paged_qjl_decode_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, case_seed)
        else:
            print(f"{head} lens={lens}", flush=True)
            paged.run_paged_decode_case(d, bits, n_seq, n_kv * g, n_kv, n_q, lens, case_seed)
