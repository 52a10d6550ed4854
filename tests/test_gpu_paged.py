"""GPU parity of the paged cache: the codes octopus_encode_paged writes into pages and the attention
octopus_attn_decode_paged computes from pages, against the oracle (which knows only logical token order).
Pages are handed out in a random order from pools larger than needed; unused pages hold garbage, so a read
of a wrong page shows."""
import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding, layout, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import DEV, check_out, sign_bits_dev, to_dev  # noqa: E402
from test_gpu_parity import compare_records, make_inputs, oracle_attention_all  # noqa: E402


def random_table(rng, n_seq, max_pages, n_pages):
    """distinct pages for every (sequence, logical tile)"""
    ids = rng.permutation(n_pages)[:n_seq * max_pages]
    return ids.reshape(n_seq, max_pages).astype(np.int32)


def pools_from_logical(cb, records, v, table, n_pages, cap):
    """records [n_seq, n_kv, T, rb], v [n_seq, n_kv, cap, d] -> (k_pool bytes, v_pool [n_pages, n_kv, 64, d])"""
    n_seq, n_kv = records.shape[:2]
    d = v.shape[-1]
    tb = cb.plan.granules * 64 * 16
    img = layout.records_to_cache(records, cb.plan.granules, cap).reshape(n_seq, n_kv, cap // 64, tb)
    k_pool = np.full((n_pages, n_kv, tb), 0xAB, dtype=np.uint8)
    v_pool = np.full((n_pages, n_kv, 64, d), 1e4, dtype=np.float32)      # garbage that would dominate an output
    for s in range(n_seq):
        for j in range(cap // 64):
            k_pool[table[s, j]] = img[s, :, j]
            v_pool[table[s, j]] = v[s, :, 64 * j:64 * j + 64]
    return k_pool, v_pool


def test_paged_decode_refuses_chunks_of_many_query_rows_where_no_many_row_kernel_serves():
    """32 or more query rows per KV head are the many-row kernel's: built up to head_dim 128, bf16 value pages."""
    cb = binding.octopus_build_codebooks(256, 3)
    q = torch.zeros((1, 11, 6, 256), dtype=torch.bfloat16, device=DEV)           # 11 queries x 3 heads per KV head
    pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, 4, 2), dtype=torch.uint8, device=DEV)
    v_pool = torch.zeros((4, 2, 64, 256), dtype=torch.bfloat16, device=DEV)
    table = torch.zeros((1, 4), dtype=torch.int32, device=DEV)
    lens = torch.tensor([200], dtype=torch.int32, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 6, 2, 11, 200), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 11, 6, 256), dtype=torch.float32, device=DEV)
    signs = torch.zeros(2 * 32, dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_attn_decode_paged(cb, q, signs, pool, v_pool, table, lens, 200, 0.1, out, ws)
    assert err.value.code == binding.EUNSUPPORTED
    # quantised value pages: the matrix-core kernel over them serves row groups, not chunks
    cb = binding.octopus_build_codebooks(128, 3)
    q = torch.zeros((1, 11, 6, 128), dtype=torch.bfloat16, device=DEV)
    pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, 4, 2), dtype=torch.uint8, device=DEV)
    vq_pool = torch.zeros(4 * 2 * 64 * binding.octopus_vq_row_bytes(128, 3, 32), dtype=torch.uint8, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 6, 2, 11, 200), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 11, 6, 128), dtype=torch.float32, device=DEV)
    signs = torch.zeros(2 * 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_attn_decode_paged_vq(cb, q, signs, pool, vq_pool, 3, 32, 2, table, lens, 200, 0.1, out, ws)
    assert err.value.code == binding.EUNSUPPORTED


@pytest.mark.parametrize("d,bits,n_qh,n_kv,n_q,lens", [
    (128, 3, 6, 2, 11, [300, 129]),          # 33 rows per KV head: one block of 128 rows, mostly padding
    (64, 4, 4, 1, 70, [1000, 64, 0]),        # 280 rows: blocks of 256 rows, two of them
    (128, 2, 8, 2, 40, [2500]),              # 160 rows: two blocks of 128; several splits
    (64, 2.5, 2, 2, 50, [200, 700])])        # 50 rows per KV head
def test_paged_decode_many_query_rows(d, bits, n_qh, n_kv, n_q, lens):
    """A chunk of queries over pages goes to the many-row kernel, as over a contiguous cache."""
    run_paged_decode_case(d, bits, len(lens), n_qh, n_kv, n_q, lens, seed=int(2000 + d + 10 * bits + n_q))


def run_paged_decode_case(d, bits, n_seq, n_qh, n_kv, n_q, lens, seed, q_dtype="bf16", spare_pages=5):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(seed)
    T = max(int(max(lens)), 1)
    cap = -(-T // 64) * 64
    max_pages = cap // 64
    n_pages = n_seq * max_pages + spare_pages
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(n_seq)])
    q = synth.queries(seed, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, q_dtype, n_q=n_q))
    v = np.zeros((n_seq, n_kv, cap, d), dtype=np.float32)
    v[:, :, :T] = vals
    table = random_table(rng, n_seq, max_pages, n_pages)
    k_pool, v_pool = pools_from_logical(cb, records, v, table, n_pages, cap)
    scale = 1.0 / np.sqrt(d)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, T), dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    binding.octopus_attn_decode_paged(cb, to_dev(q, q_dtype), sign_bits_dev(signs), torch.from_numpy(k_pool).to(DEV),
                                      to_dev(v_pool, "bf16"), torch.from_numpy(table).to(DEV),
                                      torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV), T, scale, out, ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    ref_out, _ = oracle_attention_all(plan, records, signs, q, v, lens, scale)
    worst = 0.0
    for s in range(n_seq):
        for h in range(n_qh):
            for qi in range(n_q):
                if int(lens[s]) == 0:
                    assert np.all(out[s, qi, h] == 0.0)
                else:
                    worst = max(worst, check_out(out[s, qi, h], ref_out[s, qi, h]))
    print(f"[paged attn] d={d} b={bits} lens={list(lens)}: worst out err {worst:.3g}")


@pytest.mark.parametrize("bits", [1, 1.5, 2, 2.5, 3, 4])
def test_paged_decode_gqa_ragged_d128(bits):
    run_paged_decode_case(128, bits, 3, 8, 2, 1, [0, 77, 1000], seed=int(700 + 10 * bits))


@pytest.mark.parametrize("d,bits", [(64, 2), (64, 4), (256, 2.5), (256, 3)])
def test_paged_decode_other_head_dims(d, bits):
    run_paged_decode_case(d, bits, 2, 4, 2, 3, [513, 64], seed=int(800 + d + 10 * bits))


def test_paged_decode_long_sequence_many_sequences_and_fp32_queries():
    run_paged_decode_case(128, 3, 1, 4, 1, 1, [9000], seed=901)                       # 141 pages, several splits
    rng = np.random.default_rng(902)
    run_paged_decode_case(64, 3, 70, 2, 1, 1, [int(x) for x in rng.integers(0, 300, size=70)], seed=902)
    run_paged_decode_case(128, 2, 2, 6, 2, 10, [300, 129], seed=903, q_dtype="fp32")  # 30 rows: groups of 8


def test_paged_decode_shared_prefix_pages():
    """two sequences whose first pages are the same physical pages (a common prefix)"""
    d, bits, n_kv, n_qh = 128, 3, 2, 8
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    keys, vals, signs = make_inputs(950, 2, n_kv, 320, d, "bf16")
    keys[1, :128] = keys[0, :128]                      # 2 pages of common prefix
    vals[1, :, :128] = vals[0, :, :128]
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(2)])
    table = np.array([[7, 3, 0, 9, 5], [7, 3, 1, 8, 2]], dtype=np.int32)
    k_pool, v_pool = pools_from_logical(cb, records, vals, table, 10, 320)
    lens = [320, 290]
    q = synth.queries(950, synth.Workload("t", 2, n_qh, n_kv, d, 320, bits, "bf16"))
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 2, n_qh, n_kv, 1, 320), dtype=torch.uint8, device=DEV)
    out = torch.zeros((2, 1, n_qh, d), dtype=torch.float32, device=DEV)
    scale = 1 / np.sqrt(d)
    binding.octopus_attn_decode_paged(cb, to_dev(q, "bf16"), sign_bits_dev(signs), torch.from_numpy(k_pool).to(DEV),
                                      to_dev(v_pool, "bf16"), torch.from_numpy(table).to(DEV),
                                      torch.tensor(lens, dtype=torch.int32, device=DEV), 320, scale, out, ws)
    torch.cuda.synchronize()
    ref_out, _ = oracle_attention_all(plan, records, signs, q, vals, lens, scale)
    for s in range(2):
        for h in range(n_qh):
            check_out(out.cpu().numpy()[s, 0, h], ref_out[s, 0, h])


def gather_records(cb, k_pool, table, n_seq, n_kv, cap):
    tb = cb.plan.granules * 64 * 16
    pool = k_pool.reshape(-1, n_kv, tb)
    img = np.zeros((n_seq, n_kv, cap // 64, tb), dtype=np.uint8)
    for s in range(n_seq):
        for j in range(cap // 64):
            img[s, :, j] = pool[table[s, j]]
    return layout.cache_to_records(img.reshape(-1), n_seq, n_kv, cap, cb.plan.granules, cb.plan.record_bytes)


@pytest.mark.parametrize("d,bits,dtype", [(128, 3, "bf16"), (64, 2.5, "fp32"), (256, 4, "bf16")])
def test_paged_encode_matches_the_oracle_and_leaves_other_pages_alone(d, bits, dtype):
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    n_seq, n_kv, n_tok, max_pages = 3, 2, 200, 5
    n_pages = n_seq * max_pages + 4
    rng = np.random.default_rng(int(d + 10 * bits))
    keys, _, signs = make_inputs(int(d + 10 * bits), n_seq, n_kv, n_tok, d, dtype)
    table = random_table(rng, n_seq, max_pages, n_pages)
    k_pool = torch.full((binding.octopus_paged_pool_bytes(cb, n_pages, n_kv),), 0xAB, dtype=torch.uint8, device=DEV)
    binding.octopus_encode_paged(cb, to_dev(keys, dtype), sign_bits_dev(signs), k_pool, n_pages,
                                 torch.from_numpy(table).to(DEV))
    torch.cuda.synchronize()
    pool = k_pool.cpu().numpy()
    rec, _ = gather_records(cb, pool, table, n_seq, n_kv, max_pages * 64)
    compare_records(plan, keys, signs, rec, f"paged encode d={d} b={bits}")
    tb = cb.plan.granules * 64 * 16
    used = set(table[:, :4].reshape(-1).tolist())                      # 200 tokens: tiles 0..3
    for page in range(n_pages):
        if page not in used:
            assert np.all(pool.reshape(n_pages, n_kv, tb)[page] == 0xAB)
    # the contiguous encoder writes the same bytes
    cache = torch.zeros(binding.octopus_cache_bytes(cb, n_seq, n_kv, 256), dtype=torch.uint8, device=DEV)
    binding.octopus_encode(cb, to_dev(keys, dtype), sign_bits_dev(signs), cache, 256)
    ref, _ = layout.cache_to_records(cache.cpu().numpy(), n_seq, n_kv, 256, cb.plan.granules, cb.plan.record_bytes)
    assert np.array_equal(rec[:, :, :n_tok], ref[:, :, :n_tok])


def test_paged_encode_append_then_decode_end_to_end():
    """tokens appended in three calls at unaligned positions into pages, then attention from the pages"""
    d, bits, n_seq, n_kv, n_qh, T, max_pages = 128, 3, 2, 2, 8, 300, 5
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(77)
    n_pages = 16
    keys, vals, signs = make_inputs(77, n_seq, n_kv, T, d, "bf16")
    table = random_table(rng, n_seq, max_pages, n_pages)
    tab_dev = torch.from_numpy(table).to(DEV)
    k_pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, n_pages, n_kv), dtype=torch.uint8, device=DEV)
    for lo, hi in ((0, 100), (100, 101), (101, 300)):
        binding.octopus_encode_paged(cb, to_dev(keys[:, lo:hi], "bf16"), sign_bits_dev(signs), k_pool, n_pages, tab_dev,
                                     torch.full((n_seq,), lo, dtype=torch.int32, device=DEV))
    v = np.zeros((n_seq, n_kv, max_pages * 64, d), dtype=np.float32)
    v[:, :, :T] = vals
    v_pool = np.zeros((n_pages, n_kv, 64, d), dtype=np.float32)
    for s in range(n_seq):
        for j in range(max_pages):
            v_pool[table[s, j]] = v[s, :, 64 * j:64 * j + 64]
    lens = [300, 170]
    q = synth.queries(77, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16"))
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, 1, T), dtype=torch.uint8, device=DEV)
    out = torch.zeros((n_seq, 1, n_qh, d), dtype=torch.float32, device=DEV)
    scale = 1 / np.sqrt(d)
    binding.octopus_attn_decode_paged(cb, to_dev(q, "bf16"), sign_bits_dev(signs), k_pool, to_dev(v_pool, "bf16"), tab_dev,
                                      torch.tensor(lens, dtype=torch.int32, device=DEV), T, scale, out, ws)
    torch.cuda.synchronize()
    records = np.stack([np.stack([oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h]) for h in range(n_kv)])
                        for s in range(n_seq)])
    ref_out, _ = oracle_attention_all(plan, records, signs, q, v, lens, scale)
    for s in range(n_seq):
        for h in range(n_qh):
            check_out(out.cpu().numpy()[s, 0, h], ref_out[s, 0, h])


def run_paged_hybrid_case(d, bits, n_seq, n_qh, n_kv, n_q, lens, win_lens, w_capacity, k_dtype, seed, spare_pages=4,
                          reach=None):
    """octopus_attn_decode_paged_hybrid against the oracle's dense definition over the reconstructed keys stacked
    on the window's keys (the oracle knows only logical token order): the compressed tokens' records and ALL value
    rows, the window's included, lie in randomly ordered pages."""
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(seed)
    tot = [int(a) + int(b) for a, b in zip(lens, win_lens)]
    T = max(max(tot), 1)
    cap = reach or -(-T // 64) * 64                       # tokens the block table can address (a multiple of 64)
    max_pages = cap // 64
    n_pages = n_seq * max_pages + spare_pages
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")          # keys [n_seq, T, n_kv, d]
    records = np.zeros((n_seq, n_kv, cap, plan.record_bytes), dtype=np.uint8)
    k_win = np.zeros((n_seq, n_kv, w_capacity, d), dtype=np.float32)
    for s in range(n_seq):
        L, W = int(lens[s]), int(win_lens[s])
        for h in range(n_kv):
            if L:
                records[s, h, :L] = oracle.encode(plan, keys[s, :L, h].astype(np.float64), signs[h])
            k_win[s, h, :W] = keys[s, L:L + W, h]
    q = synth.queries(seed, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16", n_q=n_q))
    v = np.zeros((n_seq, n_kv, cap, d), dtype=np.float32)
    v[:, :, :min(T, cap)] = vals[:, :, :cap]
    table = random_table(rng, n_seq, max_pages, n_pages)
    k_pool, v_pool = pools_from_logical(cb, records, v, table, n_pages, cap)
    scale = 1.0 / np.sqrt(d)
    max_len = max(int(x) for x in lens)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, max_len), dtype=torch.uint8,
                     device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    binding.octopus_attn_decode_paged_hybrid(
        cb, to_dev(q, "bf16"), sign_bits_dev(signs), torch.from_numpy(k_pool).to(DEV), to_dev(v_pool, "bf16"),
        torch.from_numpy(table).to(DEV), torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV), max_len,
        to_dev(k_win, k_dtype), torch.tensor(np.asarray(win_lens), dtype=torch.int32, device=DEV), scale, out, ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    g = n_qh // n_kv
    worst = 0.0
    for s in range(n_seq):
        L = int(lens[s])
        W = min(int(win_lens[s]), w_capacity, cap - L)          # window tokens the table cannot address are ignored
        for h in range(n_kv):
            if L + W == 0:
                assert np.all(out[s, :, h * g:(h + 1) * g] == 0.0)
                continue
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            _, ref_o = oracle.attention_hybrid(plan, records[s, h, :L], signs[h], k_win[s, h, :W], qq,
                                               v[s, h, :L + W].astype(np.float64), scale)
            ref_o = ref_o.reshape(n_q, g, d)
            for qi in range(n_q):
                for j in range(g):
                    worst = max(worst, check_out(out[s, qi, h * g + j], ref_o[qi, j]))
    print(f"[paged hybrid] d={d} b={bits} lens={list(lens)} window={list(win_lens)}: worst out err {worst:.3g}")


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_paged_hybrid_gqa_window_32_d128(bits):
    # windows that stay inside a page, straddle a page boundary, start on one, and are empty
    run_paged_hybrid_case(128, bits, 4, 8, 2, 1, [300, 100, 128, 57], [32, 32, 17, 0], 32, "bf16", seed=1700 + int(bits))


def test_paged_hybrid_other_head_dims_fp32_window_keys_and_several_queries():
    run_paged_hybrid_case(64, 2.5, 3, 4, 4, 2, [130, 0, 64], [5, 40, 64], 64, "fp32", seed=1711)
    run_paged_hybrid_case(256, 3, 2, 4, 1, 1, [200, 31], [33, 32], 48, "bf16", seed=1712)
    # 40 query rows per KV head: the many-row kernel over pages, plus the window
    run_paged_hybrid_case(128, 3, 2, 8, 2, 10, [300, 70], [32, 9], 32, "bf16", seed=1714)


def test_paged_hybrid_window_clipped_at_the_tables_reach_and_argument_errors():
    # sequence 0: 120 compressed + 30 window tokens, but two pages (128 tokens) per sequence: 8 window tokens count
    run_paged_hybrid_case(128, 3, 2, 4, 2, 1, [120, 40], [30, 20], 32, "bf16", seed=1713, reach=128)
    cb = binding.octopus_build_codebooks(128, 3)
    q = torch.zeros((1, 1, 4, 128), dtype=torch.bfloat16, device=DEV)
    pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, 4, 2), dtype=torch.uint8, device=DEV)
    v_pool = torch.zeros((4, 2, 64, 128), dtype=torch.bfloat16, device=DEV)
    table = torch.zeros((1, 4), dtype=torch.int32, device=DEV)
    lens = torch.tensor([200], dtype=torch.int32, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 4, 2, 1, 200), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 1, 4, 128), dtype=torch.float32, device=DEV)
    signs = torch.zeros(2 * 16, dtype=torch.uint8, device=DEV)
    k_win = torch.zeros((1, 2, 0, 128), dtype=torch.bfloat16, device=DEV)         # w_capacity 0
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_attn_decode_paged_hybrid(cb, q, signs, pool, v_pool, table, lens, 200, k_win, lens, 0.1, out, ws)
    assert err.value.code == binding.EINVAL


# ---- group-quantised values in pages --------------------------------------------------------------------------
def vq_pool_from_logical(vq_rows, table, n_pages, cap, fill=0x5A):
    """vq_rows [n_seq, n_kv, cap, rb] -> pool [n_pages, n_kv, 64, rb]; unused pages hold `fill`"""
    n_seq, n_kv, _, rb = vq_rows.shape
    pool = np.full((n_pages, n_kv, 64, rb), fill, dtype=np.uint8)
    for s in range(n_seq):
        for j in range(cap // 64):
            pool[table[s, j]] = vq_rows[s, :, 64 * j:64 * j + 64]
    return pool


@pytest.mark.parametrize("d,v_bits,group,dtype", [(128, 3, 32, "bf16"), (64, 2, 16, "fp32"), (256, 4, 32, "bf16")])
def test_paged_encode_values_writes_the_oracles_rows_into_the_right_pages(d, v_bits, group, dtype):
    n_seq, n_kv, n_tok, max_pages = 2, 2, 150, 4
    rng = np.random.default_rng(40 + d)
    _, vals, _ = make_inputs(41 + d, n_seq, n_kv, n_tok, d, dtype)                # vals [n_seq, n_kv, n_tok, d]
    n_pages = n_seq * max_pages + 3
    table = random_table(rng, n_seq, max_pages, n_pages)
    rb = oracle.vq_row_bytes(d, v_bits, group)
    pool = torch.full((n_pages * n_kv * 64 * rb,), 0xEE, dtype=torch.uint8, device=DEV)
    start = [0, 70]                                                               # sequence 1 appends behind 70 tokens
    v_dev = to_dev(vals, dtype).permute(0, 2, 1, 3)                               # [n_seq, n_tok, n_kv, d] view
    binding.octopus_encode_values_paged(v_dev, v_bits, group, pool, n_kv, torch.from_numpy(table).to(DEV),
                                        torch.tensor(start, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    got = pool.cpu().numpy().reshape(n_pages, n_kv, 64, rb)
    touched = np.zeros((n_pages, n_kv, 64), dtype=bool)
    for s in range(n_seq):
        for h in range(n_kv):
            ref = oracle.vq_encode(vals[s, h], v_bits, group)
            for i in range(n_tok):
                t = start[s] + i
                if t >= max_pages * 64:
                    continue                                                      # past what the table addresses: dropped
                assert np.array_equal(got[table[s, t // 64], h, t % 64], ref[i]), (s, h, i)
                touched[table[s, t // 64], h, t % 64] = True
    assert np.all(got[~touched] == 0xEE)                                          # every other row is as it was


def run_paged_vq_decode_case(d, bits, v_bits, group, n_seq, n_qh, n_kv, n_q, lens, seed, spare_pages=3):
    """octopus_attn_decode_paged_vq against the oracle's attention over its own dequantised rows; records and
    quantised rows are the oracle's, scattered over randomly ordered pages."""
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(seed)
    T = max(int(max(lens)), 1)
    cap = -(-T // 64) * 64
    max_pages = cap // 64
    n_pages = n_seq * max_pages + spare_pages
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")
    records = np.zeros((n_seq, n_kv, cap, plan.record_bytes), dtype=np.uint8)
    rb = oracle.vq_row_bytes(d, v_bits, group)
    vq_rows = np.zeros((n_seq, n_kv, cap, rb), dtype=np.uint8)
    for s in range(n_seq):
        for h in range(n_kv):
            records[s, h, :T] = oracle.encode(plan, keys[s, :, h].astype(np.float64), signs[h])
            vq_rows[s, h, :T] = oracle.vq_encode(vals[s, h], v_bits, group)
    q = synth.queries(seed, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16", n_q=n_q))
    table = random_table(rng, n_seq, max_pages, n_pages)
    k_pool, _ = pools_from_logical(cb, records, np.zeros((n_seq, n_kv, cap, d), dtype=np.float32), table, n_pages, cap)
    vq_pool = vq_pool_from_logical(vq_rows, table, n_pages, cap)
    scale = 1.0 / np.sqrt(d)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, T), dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    binding.octopus_attn_decode_paged_vq(cb, to_dev(q, "bf16"), sign_bits_dev(signs), torch.from_numpy(k_pool).to(DEV),
                                         torch.from_numpy(vq_pool.reshape(-1)).to(DEV), v_bits, group, n_kv,
                                         torch.from_numpy(table).to(DEV),
                                         torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV), T, scale, out, ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    g = n_qh // n_kv
    worst = 0.0
    for s in range(n_seq):
        L = int(lens[s])
        for h in range(n_kv):
            if L == 0:
                assert np.all(out[s, :, h * g:(h + 1) * g] == 0.0)
                continue
            v_hat = oracle.vq_decode(vq_rows[s, h, :L], d, v_bits, group)
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            _, ref_o, _ = oracle.attention(plan, records[s, h, :L], signs[h], qq, v_hat, scale)
            ref_o = ref_o.reshape(n_q, g, d)
            for qi in range(n_q):
                for j in range(g):
                    worst = max(worst, check_out(out[s, qi, h * g + j], ref_o[qi, j]))
    print(f"[paged attn-vq] d={d} b={bits} v_bits={v_bits} g={group} lens={list(lens)}: worst out err {worst:.3g}")


@pytest.mark.parametrize("d,bits,v_bits,group,n_qh,n_kv,n_q", [
    (128, 3, 3, 32, 8, 2, 1), (128, 2, 4, 32, 4, 2, 1), (128, 3, 3, 16, 4, 1, 1), (128, 4, 2, 32, 8, 1, 1),
    (64, 2.5, 3, 16, 4, 2, 1), (64, 4, 4, 32, 2, 2, 3), (256, 3, 3, 32, 4, 1, 1), (256, 1.5, 2, 32, 8, 2, 1)])
def test_paged_decode_over_quantised_value_pages(d, bits, v_bits, group, n_qh, n_kv, n_q):
    run_paged_vq_decode_case(d, bits, v_bits, group, 3, n_qh, n_kv, n_q, [300, 129, 0],
                             seed=int(1800 + d + 10 * bits + v_bits))


def test_paged_decode_over_quantised_value_pages_long_sequence_and_refusals():
    run_paged_vq_decode_case(128, 3, 3, 32, 2, 4, 1, 1, [9000, 3000], seed=1821)      # 141 pages, several items
    cb = binding.octopus_build_codebooks(128, 3)
    q = torch.zeros((1, 1, 64, 128), dtype=torch.bfloat16, device=DEV)               # 8 rows per KV head ...
    pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, 4, 8), dtype=torch.uint8, device=DEV)
    vq_pool = torch.zeros(4 * 8 * 64 * binding.octopus_vq_row_bytes(128, 3, 16), dtype=torch.uint8, device=DEV)
    table = torch.zeros((1, 4), dtype=torch.int32, device=DEV)
    lens = torch.tensor([200], dtype=torch.int32, device=DEV)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, 1, 64, 8, 1, 200), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 1, 64, 128), dtype=torch.float32, device=DEV)
    signs = torch.zeros(8 * 16, dtype=torch.uint8, device=DEV)
    assert not binding.octopus_vq_on_matrix_cores(cb, 64, 8, 1, 3, 16)               # ... x groups of 16: no such build
    with pytest.raises(binding.OctopusError) as err:
        binding.octopus_attn_decode_paged_vq(cb, q, signs, pool, vq_pool, 3, 16, 8, table, lens, 200, 0.1, out, ws)
    assert err.value.code == binding.EUNSUPPORTED


# ---- the 1-bit QJL residual in pages ------------------------------------------------------------------------------
def qjl_pool_from_logical(side_img, table, n_pages, n_seq, n_kv, cap, d, fill=0x3C):
    """contiguous side-car image (bytes, [n_seq][n_kv][cap / 64] tiles) -> pool [n_pages][n_kv] tiles"""
    tq = 64 * (d // 8 + 2)
    tiles = np.asarray(side_img, dtype=np.uint8).reshape(n_seq, n_kv, cap // 64, tq)
    pool = np.full((n_pages, n_kv, tq), fill, dtype=np.uint8)
    for s in range(n_seq):
        for j in range(cap // 64):
            pool[table[s, j]] = tiles[s, :, j]
    return pool


@pytest.mark.parametrize("d,bits,dtype", [(128, 3, "bf16"), (64, 2, "fp32"), (256, 2.5, "bf16")])
def test_paged_encode_qjl_writes_the_contiguous_encoders_bytes_into_pages(d, bits, dtype):
    """Records and side-car tiles written through the page table are byte for byte those octopus_encode_qjl writes
    into a contiguous cache (whose parity with the oracle test_gpu_qjl.py covers); other pages stay as they were."""
    from test_gpu_qjl import gpu_encode_qjl
    n_seq, n_kv, n_tok, cap = 2, 2, 150, 256
    max_pages = cap // 64
    cb = binding.octopus_build_codebooks(d, bits)
    rng = np.random.default_rng(50 + d)
    keys, _, signs = make_inputs(51 + d, n_seq, n_kv, n_tok, d, dtype)
    signs2 = synth.sign_vectors(52 + d, n_kv, d)
    start = [0, 70]
    _, _, _, cache, side = gpu_encode_qjl(cb, keys, dtype, signs, signs2, cap, start_pos=start)
    n_pages = n_seq * max_pages + 3
    table = random_table(rng, n_seq, max_pages, n_pages)
    tb, tq = cb.plan.granules * 64 * 16, 64 * (d // 8 + 2)
    k_pool = torch.full((n_pages * n_kv * tb,), 0xAB, dtype=torch.uint8, device=DEV)
    q_pool = torch.full((n_pages * n_kv * tq,), 0xCD, dtype=torch.uint8, device=DEV)
    assert q_pool.numel() == binding.octopus_qjl_bytes(cb, n_pages, n_kv, 64)
    binding.octopus_encode_qjl_paged(cb, to_dev(keys, dtype), sign_bits_dev(signs), sign_bits_dev(signs2), k_pool, q_pool,
                                     n_pages, torch.from_numpy(table).to(DEV),
                                     torch.tensor(start, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    kp = k_pool.cpu().numpy().reshape(n_pages, n_kv, tb)
    qp = q_pool.cpu().numpy().reshape(n_pages, n_kv, tq)
    kc = cache.cpu().numpy().reshape(n_seq, n_kv, max_pages, tb)
    qc = side.cpu().numpy().reshape(n_seq, n_kv, max_pages, tq)
    used = set()
    for s in range(n_seq):
        first, last = start[s] // 64, (start[s] + n_tok - 1) // 64
        for j in range(first, last + 1):
            used.add(int(table[s, j]))
            # a tile written in part keeps the pool's fill where the contiguous cache keeps its zeros: compare the
            # slots of the tokens written
            lo, hi = max(start[s], 64 * j) - 64 * j, min(start[s] + n_tok, 64 * j + 64) - 64 * j
            for h in range(n_kv):
                kt = kp[table[s, j], h].reshape(cb.plan.granules, 64, 16)
                kr = kc[s, h, j].reshape(cb.plan.granules, 64, 16)
                assert np.array_equal(kt[:, lo:hi], kr[:, lo:hi]), (s, h, j)
                nw = d // 32
                wt = qp[table[s, j], h, :nw * 256].reshape(nw, 64, 4)
                wr = qc[s, h, j, :nw * 256].reshape(nw, 64, 4)
                assert np.array_equal(wt[:, lo:hi], wr[:, lo:hi]), (s, h, j)
                gt = qp[table[s, j], h, nw * 256:].reshape(64, 2)
                gr = qc[s, h, j, nw * 256:].reshape(64, 2)
                assert np.array_equal(gt[lo:hi], gr[lo:hi]), (s, h, j)
    for pg in range(n_pages):
        if pg not in used:
            assert np.all(kp[pg] == 0xAB) and np.all(qp[pg] == 0xCD)


def run_paged_qjl_decode_case(d, bits, n_seq, n_qh, n_kv, n_q, lens, seed, spare_pages=3):
    """octopus_attn_decode_paged_qjl over the oracle's records and side-car scattered over pages, against the
    oracle's corrected attention."""
    cb = binding.octopus_build_codebooks(d, bits)
    plan = oracle.make_plan(d, bits)
    rng = np.random.default_rng(seed)
    T = max(int(max(lens)), 1)
    cap = -(-T // 64) * 64
    max_pages = cap // 64
    n_pages = n_seq * max_pages + spare_pages
    keys, vals, signs = make_inputs(seed, n_seq, n_kv, T, d, "bf16")
    signs2 = synth.sign_vectors(seed + 1000, n_kv, d)
    records = np.zeros((n_seq, n_kv, cap, plan.record_bytes), dtype=np.uint8)
    sigma = np.zeros((n_seq, n_kv, T, d), dtype=np.int8)
    gamma_r = np.zeros((n_seq, n_kv, T), dtype=np.float64)
    for s in range(n_seq):
        for h in range(n_kv):
            k = keys[s, :, h].astype(np.float64)
            records[s, h, :T] = oracle.encode(plan, k, signs[h])
            sigma[s, h], gamma_r[s, h] = oracle.qjl_encode(plan, k, signs[h], signs2[h], records[s, h, :T])
    q = synth.queries(seed, synth.Workload("t", n_seq, n_qh, n_kv, d, T, bits, "bf16", n_q=n_q))
    v = np.zeros((n_seq, n_kv, cap, d), dtype=np.float32)
    v[:, :, :T] = vals
    table = random_table(rng, n_seq, max_pages, n_pages)
    k_pool, v_pool = pools_from_logical(cb, records, v, table, n_pages, cap)
    sbits = np.packbits((sigma < 0).astype(np.uint8), axis=-1, bitorder="little")
    side = layout.qjl_from_canonical(sbits, gamma_r.astype(np.float16), cap)
    q_pool = qjl_pool_from_logical(side, table, n_pages, n_seq, n_kv, cap, d)
    scale = 1.0 / np.sqrt(d)
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, n_seq, n_qh, n_kv, n_q, T), dtype=torch.uint8, device=DEV)
    out = torch.full((n_seq, n_q, n_qh, d), float("nan"), dtype=torch.float32, device=DEV)
    binding.octopus_attn_decode_paged_qjl(cb, to_dev(q, "bf16"), sign_bits_dev(signs), sign_bits_dev(signs2),
                                          torch.from_numpy(k_pool).to(DEV), torch.from_numpy(q_pool.reshape(-1)).to(DEV),
                                          to_dev(v_pool, "bf16"), torch.from_numpy(table).to(DEV),
                                          torch.tensor(np.asarray(lens), dtype=torch.int32, device=DEV), T, scale, out, ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    g = n_qh // n_kv
    worst = 0.0
    for s in range(n_seq):
        L = int(lens[s])
        for h in range(n_kv):
            if L == 0:
                assert np.all(out[s, :, h * g:(h + 1) * g] == 0.0)
                continue
            qq = q[s, :, h * g:(h + 1) * g, :].reshape(-1, d).astype(np.float64)
            _, ref_o = oracle.attention_qjl(plan, records[s, h, :L], signs[h], signs2[h], sigma[s, h, :L],
                                            gamma_r[s, h, :L], qq, v[s, h, :L].astype(np.float64), scale)
            ref_o = ref_o.reshape(n_q, g, d)
            for qi in range(n_q):
                for j in range(g):
                    worst = max(worst, check_out(out[s, qi, h * g + j], ref_o[qi, j]))
    print(f"[paged attn-qjl] d={d} b={bits} lens={list(lens)}: worst out err {worst:.3g}")


@pytest.mark.parametrize("bits", [1, 1.5, 2, 2.5, 3, 4])
def test_paged_decode_qjl_gqa_ragged_d128(bits):
    run_paged_qjl_decode_case(128, bits, 3, 8, 2, 1, [0, 77, 1000], seed=int(1900 + 10 * bits))


def test_paged_decode_qjl_other_head_dims_and_several_queries():
    run_paged_qjl_decode_case(64, 2, 1, 3, 3, 5, [700], seed=1931)
    run_paged_qjl_decode_case(256, 4, 2, 4, 2, 1, [513, 64], seed=1932)
