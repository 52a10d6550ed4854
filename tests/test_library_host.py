"""Host-side checks of the C-ABI library that need no GPU: the shared library loads and exports what
include/octopus.h declares, plans and codebooks agree with the oracle's independent builder, and
argument errors are reported before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_21226_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ALL_BITS = (1, 1.5, 2, 2.5, 3, 4)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_21226_amd import build
        build.build(verbose=False)
    return binding.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "octopus.h")).read()
    declared = set(re.findall(r"\b(octopus_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header(lib):
    assert ctypes.sizeof(binding.Plan) == 4 * 13
    assert ctypes.sizeof(binding.Codebooks) == 4 * 13 + 4 * 2 * 64 * 4


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("bits", ALL_BITS)
def test_plan_and_codebooks_match_the_oracle(lib, d, bits):
    cb = binding.octopus_build_codebooks(d, bits)
    ref = oracle.make_plan(d, bits)
    p = cb.plan
    assert (p.head_dim, p.n_tri, p.n_class) == (d, ref.n_tri, len(ref.classes))
    assert (p.dir_bytes, p.nrm_bytes, p.record_bytes) == (ref.dir_bytes, ref.nrm_bytes, ref.record_bytes)
    assert p.granules == -(-ref.record_bytes // 16)
    for c, (nt, bd, bn) in enumerate(ref.classes):
        assert (p.class_ntri[c], p.b_dir[c], p.b_nrm[c]) == (nt, bd, bn)
        K, M = 1 << bd, 1 << bn
        # two independent Lloyd-Max builders (different quadrature, different language)
        assert np.max(np.abs(np.array(cb.c_xi[c][:K]) - ref.c_xi[c])) <= 1e-6
        assert np.max(np.abs(np.array(cb.c_rho[c][:M]) - ref.c_rho[c])) <= 1e-6
        assert np.max(np.abs(np.array(cb.b_xi[c][:K - 1]) - ref.b_xi[c]), initial=0) <= 1e-6
        assert np.max(np.abs(np.array(cb.b_rho[c][:M - 1]) - ref.b_rho[c]), initial=0) <= 1e-6
        cx = np.array(cb.c_xi[c][:K])
        assert np.all(np.diff(cx) > 0) and np.array_equal(cx, -cx[::-1])


def test_pair_codebooks_of_the_bit_allocation_sweep_match_the_oracle(lib, golden):
    """All 13 (b_dir, b_nrm) pairs of App. D's table at d = 128, up to 6 bits per index."""
    for b_dir, b_nrm, _, _ in golden("bit_split_diagonal.txt"):
        bd, bn = int(b_dir), int(b_nrm)
        cb = binding.octopus_build_codebooks_pair(128, bd, bn)
        ref = oracle.make_plan_pair(128, bd, bn)
        assert (cb.plan.dir_bytes, cb.plan.nrm_bytes, cb.plan.record_bytes) == (ref.dir_bytes, ref.nrm_bytes, ref.record_bytes)
        assert np.max(np.abs(np.array(cb.c_xi[0][:1 << bd]) - ref.c_xi[0])) <= 1e-6, (bd, bn)
        assert np.max(np.abs(np.array(cb.c_rho[0][:1 << bn]) - ref.c_rho[0])) <= 1e-6, (bd, bn)


def test_build_codebooks_errors(lib):
    cb = binding.Codebooks()
    assert lib.octopus_build_codebooks(128, 3.0, None) == binding.EINVAL
    for d, bits in [(96, 3.0), (512, 3.0), (128, 0.5), (128, 3.5), (128, 5.0), (128, 2.25)]:
        assert lib.octopus_build_codebooks(d, bits, ctypes.byref(cb)) == binding.EUNSUPPORTED
    assert lib.octopus_build_codebooks_pair(128, 7, 2, ctypes.byref(cb)) == binding.EUNSUPPORTED
    assert lib.octopus_build_codebooks_pair(128, 2, 7, ctypes.byref(cb)) == binding.EUNSUPPORTED
    assert lib.octopus_build_codebooks_pair(128, 6, 2, ctypes.byref(cb)) == binding.OK
    assert lib.octopus_build_codebooks_pair(128, 3, 3, ctypes.byref(cb)) == binding.OK
    assert cb.plan.record_bytes == 4 + oracle.stream_bytes(86, 3) + oracle.stream_bytes(43, 3)
    with pytest.raises(binding.OctopusError):
        binding.octopus_build_codebooks(100, 3)


def test_cache_bytes(lib):
    cb = binding.octopus_build_codebooks(128, 3)
    assert binding.octopus_cache_bytes(cb, 16, 8, 32768) == 16 * 8 * 32768 * 64
    assert binding.octopus_cache_bytes(cb, 1, 1, 100) == 0          # capacity must be a multiple of 64
    assert binding.octopus_cache_bytes(cb, 0, 1, 64) == 0


def test_encode_and_decode_reject_bad_arguments_before_launching(lib):
    cb = binding.octopus_build_codebooks(128, 3)
    P = ctypes.byref(cb)
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: every call below must fail validation
    null = ctypes.c_void_p(0)
    enc = lib.octopus_encode
    assert enc(P, null, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EINVAL
    assert enc(P, fake, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 100, null, null) == binding.EINVAL      # capacity
    assert enc(P, fake, 1, 1024, 1023, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EINVAL       # stride
    assert enc(P, fake, 7, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EUNSUPPORTED  # dtype
    assert enc(P, fake, 1, 1024, 1024, 128, 1, 8, 128, fake, fake, 64, null, null) == binding.EINVAL      # overflow
    assert enc(P, ctypes.c_void_p(0x1004), 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EINVAL
    assert enc(P, fake, 1, 1024, 1024, 128, 1, 8, 0, fake, fake, 64, null, null) == binding.OK             # nothing to do
    assert enc(P, fake, 1, 1024, 1024, 128, 65536, 8, 64, fake, fake, 64, null, null) == binding.EINVAL   # grid limit
    pair = binding.octopus_build_codebooks_pair(64, 3, 3)    # no kernel is built for this pair (the sweep's are d = 128)
    assert enc(ctypes.byref(pair), fake, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EUNSUPPORTED
    broken = binding.octopus_build_codebooks(128, 3)
    broken.plan.record_bytes = 57
    assert enc(ctypes.byref(broken), fake, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, null) == binding.EINVAL

    rnd = lib.octopus_encode_rounding
    assert rnd(P, fake, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, 5, null) == binding.EINVAL    # mode
    assert rnd(P, fake, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, -1, null) == binding.EINVAL
    assert rnd(P, null, 1, 1024, 1024, 128, 1, 8, 64, fake, fake, 64, null, 2, null) == binding.EINVAL
    assert rnd(P, fake, 1, 1024, 1024, 128, 1, 8, 0, fake, fake, 64, null, 2, null) == binding.OK         # nothing to do

    dec = lib.octopus_attn_decode
    ws = binding.octopus_attn_decode_workspace(cb, 2, 32, 8, 1, 4096)
    assert ws > 0 and ws % 256 == 0
    assert binding.octopus_attn_decode_workspace(cb, 2, 30, 8, 1, 4096) == 0    # heads not divisible
    args = lambda **k: [k.get("cb", P), k.get("q", fake), 1, 2, k.get("nq_heads", 32), 8, 1, fake, fake,
                        k.get("cap", 4096), fake, 1, fake, k.get("max_len", 4096), ctypes.c_float(k.get("scale", 0.1)),
                        fake, null, k.get("ws", ctypes.c_void_p(0x10000)), k.get("ws_bytes", ws), null]
    assert dec(*args(q=null)) == binding.EINVAL
    assert dec(*args(nq_heads=30)) == binding.EINVAL
    assert dec(*args(max_len=8192)) == binding.EINVAL
    assert dec(*args(ws=null)) == binding.EWORKSPACE
    assert dec(*args(ws=ctypes.c_void_p(0x10010))) == binding.EWORKSPACE        # misaligned
    assert dec(*args(ws_bytes=ws - 1)) == binding.EWORKSPACE
    assert dec(*args(scale=float("nan"))) == binding.EINVAL
    assert binding.strerror(binding.EWORKSPACE).startswith("workspace")

    # the variant with the QJL residual: same validation, plus its own arguments
    decq = lib.octopus_attn_decode_qjl
    argsq = lambda **k: [P, fake, 1, 2, 32, 8, 1, fake, k.get("signs2", fake), fake, k.get("qjl", fake), 4096, fake,
                         k.get("v_dtype", 1), fake, k.get("max_len", 4096), ctypes.c_float(0.1), fake, null,
                         k.get("ws", ctypes.c_void_p(0x10000)), k.get("ws_bytes", ws), null]
    assert decq(*argsq(signs2=null)) == binding.EINVAL
    assert decq(*argsq(qjl=null)) == binding.EINVAL
    assert decq(*argsq(qjl=ctypes.c_void_p(0x1002))) == binding.EINVAL          # misaligned side-car
    assert decq(*argsq(v_dtype=0)) == binding.EUNSUPPORTED                      # fp32 values
    assert decq(*argsq(max_len=8192)) == binding.EINVAL
    assert decq(*argsq(ws_bytes=ws - 1)) == binding.EWORKSPACE


def test_qjl_sidecar_layout_round_trip():
    from paper_2605_21226_amd import layout
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 256, (2, 3, 100, 16), dtype=np.uint8)
    g = rng.random((2, 3, 100)).astype(np.float16)
    img = layout.qjl_from_canonical(bits, g, 128)
    assert img.size == 2 * 3 * 128 * (128 // 8 + 2)
    b2, g2 = layout.qjl_to_canonical(img, 2, 3, 128, 128)
    assert np.array_equal(b2[:, :, :100], bits) and np.array_equal(g2[:, :, :100], g)
    assert not b2[:, :, 100:].any() and not g2[:, :, 100:].any()
    # word w of key t in tile T sits at byte ((T * tile_bytes) + (w * 64 + t) * 4): bit 0 of byte 4 of key 1
    one = np.zeros((1, 1, 64, 16), dtype=np.uint8)
    one[0, 0, 1, 4] = 1
    img1 = layout.qjl_from_canonical(one, np.zeros((1, 1, 64), dtype=np.float16), 64)
    assert np.flatnonzero(img1).tolist() == [(1 * 64 + 1) * 4]


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "liboctopus.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load()


def test_encode_refuses_a_codebook_too_fine_for_the_seed_grid():
    """Host-side validation only (nothing is launched): two boundaries of C_xi within one grid cell."""
    import ctypes
    lib = binding.load()
    cb = binding.octopus_build_codebooks(128, 3)
    bad = binding.Codebooks.from_buffer_copy(cb)
    bad.c_xi[0][8] = bad.c_xi[0][7] + 1e-4          # boundaries 7 and 8 now share a cell
    bad.c_xi[0][9] = bad.c_xi[0][7] + 2e-4
    dummy = ctypes.c_void_p(0x1000)                  # 16-byte aligned, never dereferenced on the host
    args = (dummy, binding.DTYPE_BF16, 0, 1024, 128, 1, 1, 64, dummy, dummy, 64, None, None)
    assert lib.octopus_encode(ctypes.byref(bad), *args) == binding.EUNSUPPORTED
    bad2 = binding.Codebooks.from_buffer_copy(cb)
    bad2.c_xi[0][3], bad2.c_xi[0][4] = bad2.c_xi[0][4], bad2.c_xi[0][3]   # not ascending
    assert lib.octopus_encode(ctypes.byref(bad2), *args) == binding.EUNSUPPORTED
    # the encoder keeps one quadrant of the direction table: C_xi must be antisymmetric to the bit
    bad3 = binding.Codebooks.from_buffer_copy(cb)
    bad3.c_xi[0][15] = float(np.nextafter(np.float32(bad3.c_xi[0][15]), np.float32(2.0)))
    assert bad3.c_xi[0][15] != -bad3.c_xi[0][0]
    assert lib.octopus_encode(ctypes.byref(bad3), *args) == binding.EUNSUPPORTED


def test_which_kernel_serves_quantised_values():
    """Host-side query used by bench.py to name the kernel it measured."""
    cb = binding.octopus_build_codebooks(128, 3)
    assert binding.octopus_vq_on_matrix_cores(cb, 32, 8, 1, 3, 32)          # GQA 4, groups of 32: matrix cores
    assert binding.octopus_vq_on_matrix_cores(cb, 32, 8, 1, 3, 16)          # groups of 16: the four-wavefront build fits
    assert binding.octopus_vq_on_matrix_cores(cb, 64, 8, 1, 3, 32)          # GQA 8 likewise
    assert not binding.octopus_vq_on_matrix_cores(cb, 64, 8, 1, 3, 16)      # eight rows x groups of 16: no build fits LDS
    assert not binding.octopus_vq_on_matrix_cores(cb, 32, 8, 1, 5, 32)      # not a value format
    assert not binding.octopus_vq_on_matrix_cores(cb, 30, 8, 1, 3, 32)      # heads not divisible
    assert binding.octopus_vq_on_matrix_cores(binding.octopus_build_codebooks(64, 2), 8, 8, 1, 2, 16)


def test_every_built_codebook_is_antisymmetric():
    """What the encoder's quadrant table relies on: c_xi[K - 1 - k] == -c_xi[k] exactly, for every bit width
    and every pair of the App. D sweep."""
    books = [binding.octopus_build_codebooks(d, b) for d in (64, 128, 256) for b in (1, 1.5, 2, 2.5, 3, 4)]
    books += [binding.octopus_build_codebooks_pair(128, bd, bn) for bd in range(1, 7) for bn in range(1, 7)
              if 2 * bd + bn in (5, 6, 7, 8, 9, 10, 11, 12, 13, 14) and bd <= 6 and bn <= 6 and (bd, bn) in
              ((1, 3), (2, 2), (3, 1), (1, 5), (2, 4), (3, 3), (4, 2), (5, 1), (2, 6), (3, 5), (4, 4), (5, 3), (6, 2))]
    assert len(books) == 18 + 13
    for cb in books:
        for c in range(cb.plan.n_class):
            K = 1 << cb.plan.b_dir[c]
            xi = np.array([cb.c_xi[c][k] for k in range(K)], dtype=np.float32)
            assert np.array_equal(xi[::-1], -xi), (cb.plan.head_dim, c, K)


def test_value_codec_sizes_and_argument_checks(lib):
    for d in (64, 128, 256):
        for b in (2, 3, 4):
            for g in (16, 32):
                assert binding.octopus_vq_row_bytes(d, b, g) == oracle.vq_row_bytes(d, b, g) == b * d // 8 + 8 * d // g
    assert binding.octopus_vq_row_bytes(128, 1, 32) == 0 and binding.octopus_vq_row_bytes(128, 3, 64) == 0
    assert binding.octopus_vq_bytes(128, 3, 32, 16, 8, 32768) == 80 * 16 * 8 * 32768
    assert binding.octopus_vq_bytes(128, 3, 32, 0, 8, 64) == 0
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    enc = lib.octopus_encode_values
    assert enc(null, 1, 1024, 1024, 128, 1, 8, 64, 128, 3, 32, fake, 64, null, null) == binding.EINVAL
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 64, 128, 3, 32, null, 64, null, null) == binding.EINVAL
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 64, 128, 5, 32, fake, 64, null, null) == binding.EUNSUPPORTED
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 64, 96, 3, 32, fake, 64, null, null) == binding.EUNSUPPORTED
    assert enc(fake, 7, 1024, 1024, 128, 1, 8, 64, 128, 3, 32, fake, 64, null, null) == binding.EUNSUPPORTED
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 128, 128, 3, 32, fake, 64, null, null) == binding.EINVAL    # overflow
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 64, 128, 3, 32, ctypes.c_void_p(0x1008), 64, null, null) == binding.EINVAL
    assert enc(fake, 1, 1024, 1024, 128, 1, 8, 0, 128, 3, 32, fake, 64, null, null) == binding.OK          # nothing to do
    # the launch's own limits: one sequence per grid z, at most 4096 (KV head, group) pairs per token
    assert enc(fake, 1, 1024, 1024, 128, 65536, 8, 0, 128, 3, 32, fake, 64, null, null) == binding.EINVAL
    assert enc(fake, 1, 1024, 1024, 128, 1, 513, 0, 128, 3, 16, fake, 64, null, null) == binding.EINVAL
    assert enc(fake, 1, 1024, 1024, 128, 65535, 512, 0, 128, 3, 16, fake, 64, null, null) == binding.OK
    cb = binding.octopus_build_codebooks(128, 3)
    ws = binding.octopus_attn_decode_workspace(cb, 2, 32, 8, 1, 4096)
    dec = lib.octopus_attn_decode_vq
    args = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, fake, 4096, k.get("vq", fake), k.get("bits", 3),
                        k.get("group", 32), fake, 4096, ctypes.c_float(0.1), fake, null, ctypes.c_void_p(0x10000),
                        k.get("ws_bytes", ws), null]
    assert dec(*args(vq=null)) == binding.EINVAL
    assert dec(*args(bits=1)) == binding.EUNSUPPORTED
    assert dec(*args(group=8)) == binding.EUNSUPPORTED
    assert dec(*args(ws_bytes=ws - 1)) == binding.EWORKSPACE


def test_hybrid_decode_argument_checks(lib):
    cb = binding.octopus_build_codebooks(128, 3)
    ws = binding.octopus_attn_decode_workspace(cb, 2, 32, 8, 1, 4096)
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    dec = lib.octopus_attn_decode_hybrid
    args = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, fake, 4096, fake, 1, fake, 4096,
                        k.get("k_window", fake), k.get("k_dtype", 1), k.get("w_capacity", 32), k.get("win_lens", fake),
                        ctypes.c_float(0.1), fake, null, ctypes.c_void_p(0x10000), k.get("ws_bytes", ws), null]
    assert dec(*args(k_window=null)) == binding.EINVAL
    assert dec(*args(win_lens=null)) == binding.EINVAL
    assert dec(*args(w_capacity=0)) == binding.EINVAL
    assert dec(*args(k_dtype=5)) == binding.EUNSUPPORTED
    assert dec(*args(ws_bytes=ws - 1)) == binding.EWORKSPACE


def test_paged_cache_sizes_and_argument_checks(lib):
    cb = binding.octopus_build_codebooks(128, 3)
    assert binding.octopus_paged_pool_bytes(cb, 10, 8) == 10 * 8 * 64 * cb.plan.granules * 16
    assert binding.octopus_paged_pool_bytes(cb, 0, 8) == 0
    ws = binding.octopus_attn_decode_workspace(cb, 2, 32, 8, 1, 4096)
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    dec = lib.octopus_attn_decode_paged
    dargs = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, k.get("k_pool", fake), k.get("v_pool", fake),
                         k.get("n_pages", 128), k.get("table", fake), k.get("max_pages", 64), fake,
                         k.get("max_len", 4096), ctypes.c_float(0.1), fake, ctypes.c_void_p(0x10000),
                         k.get("ws_bytes", ws), null]
    assert dec(*dargs(k_pool=null)) == binding.EINVAL
    assert dec(*dargs(v_pool=null)) == binding.EINVAL
    assert dec(*dargs(table=null)) == binding.EINVAL
    assert dec(*dargs(n_pages=0)) == binding.EINVAL
    assert dec(*dargs(max_pages=0)) == binding.EINVAL
    assert dec(*dargs(max_len=4097)) == binding.EINVAL            # beyond what 64 pages of 64 tokens hold
    assert dec(*dargs(k_pool=ctypes.c_void_p(0x1004))) == binding.EINVAL
    assert dec(*dargs(ws_bytes=ws - 1)) == binding.EWORKSPACE
    hyb = lib.octopus_attn_decode_paged_hybrid
    hargs = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, k.get("k_pool", fake), fake, 128, fake, 64, fake,
                         k.get("max_len", 4096), k.get("k_window", fake), k.get("k_dtype", 1), k.get("w_capacity", 32),
                         k.get("win_lens", fake), ctypes.c_float(0.1), fake, ctypes.c_void_p(0x10000),
                         k.get("ws_bytes", ws), null]
    assert hyb(*hargs(k_window=null)) == binding.EINVAL
    assert hyb(*hargs(win_lens=null)) == binding.EINVAL
    assert hyb(*hargs(w_capacity=0)) == binding.EINVAL
    assert hyb(*hargs(k_dtype=5)) == binding.EUNSUPPORTED
    assert hyb(*hargs(k_pool=null)) == binding.EINVAL
    assert hyb(*hargs(max_len=4097)) == binding.EINVAL
    assert hyb(*hargs(ws_bytes=ws - 1)) == binding.EWORKSPACE
    pq = lib.octopus_attn_decode_paged_qjl
    qargs = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, k.get("signs2", fake), k.get("k_pool", fake),
                         k.get("qjl_pool", fake), fake, 128, k.get("table", fake), 64, fake, k.get("max_len", 4096),
                         ctypes.c_float(0.1), fake, ctypes.c_void_p(0x10000), k.get("ws_bytes", ws), null]
    assert pq(*qargs(signs2=null)) == binding.EINVAL
    assert pq(*qargs(qjl_pool=null)) == binding.EINVAL
    assert pq(*qargs(qjl_pool=ctypes.c_void_p(0x1002))) == binding.EINVAL
    assert pq(*qargs(table=null)) == binding.EINVAL
    assert pq(*qargs(max_len=4097)) == binding.EINVAL
    assert pq(*qargs(ws_bytes=ws - 1)) == binding.EWORKSPACE
    eq = lib.octopus_encode_qjl_paged
    qeargs = lambda **k: [ctypes.byref(cb), fake, 1, 8 * 1024, 1024, 128, 2, 8, k.get("n_new", 64), fake,
                          k.get("signs2", fake), fake, k.get("qjl_pool", fake), k.get("n_pages", 128), fake, 4, null, null]
    assert eq(*qeargs(signs2=null)) == binding.EINVAL
    assert eq(*qeargs(qjl_pool=null)) == binding.EINVAL
    assert eq(*qeargs(n_pages=0)) == binding.EINVAL
    assert eq(*qeargs(n_new=257)) == binding.EINVAL
    assert eq(*qeargs(n_new=0)) == binding.OK
    pvq = lib.octopus_attn_decode_paged_vq
    vargs = lambda **k: [ctypes.byref(cb), fake, 1, 2, 32, 8, 1, fake, k.get("k_pool", fake), k.get("vq_pool", fake),
                         k.get("bits", 3), k.get("group", 32), 128, k.get("table", fake), 64, fake, k.get("max_len", 4096),
                         ctypes.c_float(0.1), fake, ctypes.c_void_p(0x10000), k.get("ws_bytes", ws), null]
    assert pvq(*vargs(vq_pool=null)) == binding.EINVAL
    assert pvq(*vargs(table=null)) == binding.EINVAL
    assert pvq(*vargs(bits=0)) == binding.EUNSUPPORTED
    assert pvq(*vargs(bits=5)) == binding.EUNSUPPORTED
    assert pvq(*vargs(group=8)) == binding.EUNSUPPORTED
    assert pvq(*vargs(max_len=4097)) == binding.EINVAL
    assert pvq(*vargs(ws_bytes=ws - 1)) == binding.EWORKSPACE
    pve = lib.octopus_encode_values_paged
    veargs = lambda **k: [fake, 1, 1024, 1024, 128, 1, 8, k.get("n_new", 64), 128, k.get("bits", 3), 32,
                          k.get("pool", fake), k.get("n_pages", 16), k.get("table", fake), 4, null, null]
    assert pve(*veargs(pool=null)) == binding.EINVAL
    assert pve(*veargs(table=null)) == binding.EINVAL
    assert pve(*veargs(n_pages=0)) == binding.EINVAL
    assert pve(*veargs(bits=5)) == binding.EUNSUPPORTED
    assert pve(*veargs(n_new=257)) == binding.EINVAL              # more rows than 4 pages hold, no start positions
    assert pve(*veargs(n_new=0)) == binding.OK
    enc = lib.octopus_encode_paged
    eargs = lambda **k: [ctypes.byref(cb), fake, 1, 8 * 1024, 1024, 128, 2, 8, k.get("n_new", 64), fake,
                         k.get("k_pool", fake), k.get("n_pages", 128), k.get("table", fake), k.get("max_pages", 4),
                         k.get("start", null), null]
    assert enc(*eargs(k_pool=null)) == binding.EINVAL
    assert enc(*eargs(table=null)) == binding.EINVAL
    assert enc(*eargs(n_pages=0)) == binding.EINVAL
    assert enc(*eargs(n_new=257)) == binding.EINVAL               # more tokens than 4 pages hold, no start positions
    assert enc(*eargs(n_new=0)) == binding.OK                     # nothing to do, nothing launched
