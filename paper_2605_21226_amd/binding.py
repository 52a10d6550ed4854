"""ctypes binding of liboctopus.so: argument marshalling only.

Every step of the hot path runs in the HIP kernels behind the C ABI declared
in include/octopus.h; torch is used for device memory and streams.  There is no
CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liboctopus.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
DTYPE_F32, DTYPE_BF16 = 0, 1
MAX_LEVELS = 64
TILE = 64

EXPORTS = ("octopus_build_codebooks", "octopus_build_codebooks_pair", "octopus_cache_bytes", "octopus_encode",
           "octopus_attn_decode_workspace", "octopus_attn_decode", "octopus_profile_events", "octopus_strerror",
           "octopus_qjl_bytes", "octopus_encode_qjl", "octopus_attn_decode_qjl",
           "octopus_encode_rounding", "octopus_vq_row_bytes", "octopus_vq_bytes", "octopus_encode_values",
           "octopus_attn_decode_vq", "octopus_attn_decode_hybrid",
           "octopus_paged_pool_bytes", "octopus_encode_paged", "octopus_attn_decode_paged",
           "octopus_attn_decode_paged_hybrid", "octopus_encode_values_paged", "octopus_attn_decode_paged_vq",
           "octopus_encode_qjl_paged", "octopus_attn_decode_paged_qjl",
           "octopus_attn_decode_static", "octopus_probe_read", "octopus_vq_on_matrix_cores")


class Plan(ctypes.Structure):
    _fields_ = [
        ("head_dim", ctypes.c_int32),
        ("n_tri", ctypes.c_int32),
        ("n_class", ctypes.c_int32),
        ("class_ntri", ctypes.c_int32 * 2),
        ("b_dir", ctypes.c_int32 * 2),
        ("b_nrm", ctypes.c_int32 * 2),
        ("dir_bytes", ctypes.c_int32),
        ("nrm_bytes", ctypes.c_int32),
        ("record_bytes", ctypes.c_int32),
        ("granules", ctypes.c_int32),
    ]


class Codebooks(ctypes.Structure):
    _fields_ = [
        ("plan", Plan),
        ("c_xi", (ctypes.c_float * MAX_LEVELS) * 2),
        ("b_xi", (ctypes.c_float * MAX_LEVELS) * 2),
        ("c_rho", (ctypes.c_float * MAX_LEVELS) * 2),
        ("b_rho", (ctypes.c_float * MAX_LEVELS) * 2),
    ]


class OctopusError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def load():
    """Load liboctopus.so (built in-tree by paper_2605_21226_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2605_21226_amd.build` "
                           "(or __graft_entry__.build()); there is no fallback path")
    try:
        import torch  # noqa: F401  (its HIP runtime must be the one the library binds to)
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    CB = ctypes.POINTER(Codebooks)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.octopus_build_codebooks.argtypes = [i32, f32, CB]
    lib.octopus_build_codebooks.restype = ctypes.c_int
    lib.octopus_build_codebooks_pair.argtypes = [i32, i32, i32, CB]
    lib.octopus_build_codebooks_pair.restype = ctypes.c_int
    lib.octopus_cache_bytes.argtypes = [CB, i32, i32, i64]
    lib.octopus_cache_bytes.restype = ctypes.c_size_t
    lib.octopus_encode.argtypes = [CB, vp, i32, i64, i64, i64, i32, i32, i32, vp, vp, i64, vp, vp]
    lib.octopus_encode.restype = ctypes.c_int
    lib.octopus_qjl_bytes.argtypes = [CB, i32, i32, i64]
    lib.octopus_qjl_bytes.restype = ctypes.c_size_t
    lib.octopus_encode_rounding.argtypes = [CB, vp, i32, i64, i64, i64, i32, i32, i32, vp, vp, i64, vp, i32, vp]
    lib.octopus_encode_rounding.restype = ctypes.c_int
    lib.octopus_vq_row_bytes.argtypes = [i32, i32, i32]
    lib.octopus_vq_row_bytes.restype = ctypes.c_size_t
    lib.octopus_vq_bytes.argtypes = [i32, i32, i32, i32, i32, i64]
    lib.octopus_vq_bytes.restype = ctypes.c_size_t
    lib.octopus_encode_values.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, i32, i32, vp, i64, vp, vp]
    lib.octopus_encode_values.restype = ctypes.c_int
    lib.octopus_attn_decode_vq.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, i64, vp, i32, i32, vp, i64, f32,
                                           vp, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_vq.restype = ctypes.c_int
    lib.octopus_encode_qjl.argtypes = [CB, vp, i32, i64, i64, i64, i32, i32, i32, vp, vp, vp, vp, i64, vp, vp]
    lib.octopus_encode_qjl.restype = ctypes.c_int
    lib.octopus_attn_decode_workspace.argtypes = [CB, i32, i32, i32, i32, i64]
    lib.octopus_attn_decode_workspace.restype = ctypes.c_size_t
    lib.octopus_attn_decode.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, i64, vp, i32, vp, i64, f32, vp, vp,
                                        vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode.restype = ctypes.c_int
    lib.octopus_attn_decode_static.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, i64, vp, i32, vp, i64, f32, vp, vp,
                                               vp]
    lib.octopus_attn_decode_static.restype = ctypes.c_int
    lib.octopus_attn_decode_qjl.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, i64, vp, i32, vp, i64, f32,
                                            vp, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_qjl.restype = ctypes.c_int
    lib.octopus_attn_decode_hybrid.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, i64, vp, i32, vp, i64, vp, i32,
                                               i64, vp, f32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_hybrid.restype = ctypes.c_int
    lib.octopus_paged_pool_bytes.argtypes = [CB, i32, i32]
    lib.octopus_paged_pool_bytes.restype = ctypes.c_size_t
    lib.octopus_encode_paged.argtypes = [CB, vp, i32, i64, i64, i64, i32, i32, i32, vp, vp, i32, vp, i32, vp, vp]
    lib.octopus_encode_paged.restype = ctypes.c_int
    lib.octopus_attn_decode_paged.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, vp, i32, vp, i32, vp, i64, f32,
                                              vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_paged.restype = ctypes.c_int
    lib.octopus_attn_decode_paged_hybrid.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, vp, i32, vp, i32, vp, i64,
                                                     vp, i32, i64, vp, f32, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_paged_hybrid.restype = ctypes.c_int
    lib.octopus_encode_values_paged.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, vp]
    lib.octopus_encode_values_paged.restype = ctypes.c_int
    lib.octopus_attn_decode_paged_vq.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, vp, i32, i32, i32, vp, i32, vp,
                                                 i64, f32, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_paged_vq.restype = ctypes.c_int
    lib.octopus_encode_qjl_paged.argtypes = [CB, vp, i32, i64, i64, i64, i32, i32, i32, vp, vp, vp, vp, i32, vp, i32, vp, vp]
    lib.octopus_encode_qjl_paged.restype = ctypes.c_int
    lib.octopus_attn_decode_paged_qjl.argtypes = [CB, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, i32, vp,
                                                  i64, f32, vp, vp, ctypes.c_size_t, vp]
    lib.octopus_attn_decode_paged_qjl.restype = ctypes.c_int
    lib.octopus_vq_on_matrix_cores.argtypes = [ctypes.POINTER(Codebooks), i32, i32, i32, i32, i32]
    lib.octopus_vq_on_matrix_cores.restype = ctypes.c_int
    lib.octopus_probe_read.argtypes = [vp, ctypes.c_size_t, i32, i32, vp, vp]
    lib.octopus_probe_read.restype = ctypes.c_int
    lib.octopus_profile_events.argtypes = [vp, vp]
    lib.octopus_profile_events.restype = ctypes.c_int
    lib.octopus_strerror.argtypes = [ctypes.c_int]
    lib.octopus_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def strerror(code):
    return load().octopus_strerror(int(code)).decode()


def _check(code, where):
    if code != OK:
        raise OctopusError(code, where)


def octopus_build_codebooks(head_dim, bits):
    cb = Codebooks()
    _check(load().octopus_build_codebooks(int(head_dim), float(bits), ctypes.byref(cb)), "octopus_build_codebooks")
    return cb


def octopus_build_codebooks_pair(head_dim, b_dir, b_nrm):
    cb = Codebooks()
    _check(load().octopus_build_codebooks_pair(int(head_dim), int(b_dir), int(b_nrm), ctypes.byref(cb)),
           "octopus_build_codebooks_pair")
    return cb


def octopus_cache_bytes(cb, n_seq, n_kv_heads, t_capacity):
    return int(load().octopus_cache_bytes(ctypes.byref(cb), int(n_seq), int(n_kv_heads), int(t_capacity)))


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def octopus_encode(cb, keys, signs, cache, t_capacity, start_pos=None, stream=None):
    """keys: device tensor [n_seq, n_new, n_kv_heads, d] (any strides with a contiguous last dim),
    fp32 or bf16; signs: device uint8 [n_kv_heads, d/8]; cache: device uint8 buffer of
    octopus_cache_bytes(...) bytes; start_pos: device int32 [n_seq] or None."""
    assert keys.dim() == 4 and keys.stride(3) == 1
    n_seq, n_new, n_kv, _ = keys.shape
    code = load().octopus_encode(ctypes.byref(cb), _ptr(keys), _dtype_code(keys), keys.stride(0), keys.stride(1),
                                 keys.stride(2), n_seq, n_kv, n_new, _ptr(signs), _ptr(cache), int(t_capacity),
                                 _ptr(start_pos), _stream_ptr(stream))
    _check(code, "octopus_encode")


def octopus_qjl_bytes(cb, n_seq, n_kv_heads, t_capacity):
    return int(load().octopus_qjl_bytes(ctypes.byref(cb), int(n_seq), int(n_kv_heads), int(t_capacity)))


ROUND_SEED, ROUND_LOCAL_3X3, ROUND_FULL, ROUND_INDEPENDENT, ROUND_LOCAL_2X2 = 0, 1, 2, 3, 4


def octopus_encode_rounding(cb, keys, signs, cache, t_capacity, rounding, start_pos=None, stream=None):
    """octopus_encode with one of the rounding modes ROUND_* (App. E)."""
    assert keys.dim() == 4 and keys.stride(3) == 1
    n_seq, n_new, n_kv, _ = keys.shape
    code = load().octopus_encode_rounding(ctypes.byref(cb), _ptr(keys), _dtype_code(keys), keys.stride(0),
                                          keys.stride(1), keys.stride(2), n_seq, n_kv, n_new, _ptr(signs), _ptr(cache),
                                          int(t_capacity), _ptr(start_pos), int(rounding), _stream_ptr(stream))
    _check(code, "octopus_encode_rounding")


def octopus_encode_qjl(cb, keys, signs, signs2, cache, qjl, t_capacity, start_pos=None, stream=None):
    """octopus_encode plus the QJL side-car; signs2: device uint8 [n_kv_heads, d/8]; qjl: device uint8 buffer of
    octopus_qjl_bytes(...) bytes."""
    assert keys.dim() == 4 and keys.stride(3) == 1
    n_seq, n_new, n_kv, _ = keys.shape
    code = load().octopus_encode_qjl(ctypes.byref(cb), _ptr(keys), _dtype_code(keys), keys.stride(0), keys.stride(1),
                                     keys.stride(2), n_seq, n_kv, n_new, _ptr(signs), _ptr(signs2), _ptr(cache),
                                     _ptr(qjl), int(t_capacity), _ptr(start_pos), _stream_ptr(stream))
    _check(code, "octopus_encode_qjl")


def octopus_attn_decode_workspace(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len):
    return int(load().octopus_attn_decode_workspace(ctypes.byref(cb), int(n_seq), int(n_q_heads), int(n_kv_heads),
                                                    int(n_q), int(max_len)))


def octopus_attn_decode(cb, q, signs, cache, t_capacity, v, seq_lens, max_len, scale, out, workspace,
                        scores_out=None, stream=None):
    """q: device [n_seq, n_q, n_q_heads, d] contiguous; v: device [n_seq, n_kv_heads, t_capacity, d]
    contiguous; seq_lens: device int32 [n_seq]; out: device fp32 [n_seq, n_q, n_q_heads, d];
    workspace: device uint8 buffer; scores_out: device fp32 [n_seq, n_q, n_q_heads, t_capacity] or None."""
    assert q.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_kv = v.shape[1]
    code = load().octopus_attn_decode(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q, _ptr(signs),
                                      _ptr(cache), int(t_capacity), _ptr(v), _dtype_code(v), _ptr(seq_lens),
                                      int(max_len), float(scale), _ptr(out), _ptr(scores_out), _ptr(workspace),
                                      int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode")


def octopus_attn_decode_static(cb, q, signs, cache, t_capacity, v, seq_lens, max_len, scale, out, scores_out=None,
                               stream=None):
    """octopus_attn_decode without a workspace: the library's static scratch array serves (no allocation)."""
    assert q.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_kv = v.shape[1]
    code = load().octopus_attn_decode_static(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                             _ptr(signs), _ptr(cache), int(t_capacity), _ptr(v), _dtype_code(v),
                                             _ptr(seq_lens), int(max_len), float(scale), _ptr(out), _ptr(scores_out),
                                             _stream_ptr(stream))
    _check(code, "octopus_attn_decode_static")


def octopus_attn_decode_qjl(cb, q, signs, signs2, cache, qjl, t_capacity, v, seq_lens, max_len, scale, out, workspace,
                            scores_out=None, stream=None):
    """octopus_attn_decode with the QJL-corrected score; signs2 and qjl as for octopus_encode_qjl; v: bf16."""
    assert q.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_kv = v.shape[1]
    code = load().octopus_attn_decode_qjl(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                          _ptr(signs), _ptr(signs2), _ptr(cache), _ptr(qjl), int(t_capacity), _ptr(v),
                                          _dtype_code(v), _ptr(seq_lens), int(max_len), float(scale), _ptr(out),
                                          _ptr(scores_out), _ptr(workspace),
                                          int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode_qjl")


def octopus_vq_row_bytes(head_dim, bits, group):
    return int(load().octopus_vq_row_bytes(int(head_dim), int(bits), int(group)))


def octopus_vq_bytes(head_dim, bits, group, n_seq, n_kv_heads, t_capacity):
    return int(load().octopus_vq_bytes(int(head_dim), int(bits), int(group), int(n_seq), int(n_kv_heads),
                                       int(t_capacity)))


def octopus_encode_values(v, bits, group, vq, t_capacity, start_pos=None, stream=None):
    """v: device [n_seq, n_new, n_kv_heads, d] (fp32 or bf16, channels contiguous); vq: device uint8 buffer of
    octopus_vq_bytes(...) bytes."""
    assert v.dim() == 4 and v.stride(3) == 1
    n_seq, n_new, n_kv, d = v.shape
    code = load().octopus_encode_values(_ptr(v), _dtype_code(v), v.stride(0), v.stride(1), v.stride(2), n_seq, n_kv,
                                        n_new, d, int(bits), int(group), _ptr(vq), int(t_capacity), _ptr(start_pos),
                                        _stream_ptr(stream))
    _check(code, "octopus_encode_values")


def octopus_attn_decode_vq(cb, q, signs, cache, t_capacity, vq, v_bits, v_group, n_kv_heads, seq_lens, max_len, scale,
                           out, workspace, scores_out=None, stream=None):
    """octopus_attn_decode over the quantised value rows vq (octopus_encode_values)."""
    assert q.is_contiguous() and out.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    code = load().octopus_attn_decode_vq(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, int(n_kv_heads), n_q,
                                         _ptr(signs), _ptr(cache), int(t_capacity), _ptr(vq), int(v_bits), int(v_group),
                                         _ptr(seq_lens), int(max_len), float(scale), _ptr(out), _ptr(scores_out),
                                         _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                         _stream_ptr(stream))
    _check(code, "octopus_attn_decode_vq")


def octopus_attn_decode_hybrid(cb, q, signs, cache, t_capacity, v, seq_lens, max_len, k_window, win_lens, scale, out,
                               workspace, scores_out=None, stream=None):
    """octopus_attn_decode plus a native-precision window: k_window device [n_seq, n_kv_heads, w_capacity, d]
    contiguous (fp32 or bf16), win_lens device int32 [n_seq]; the window's values follow the compressed tokens'
    in v."""
    assert q.is_contiguous() and v.is_contiguous() and out.is_contiguous() and k_window.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_kv = v.shape[1]
    code = load().octopus_attn_decode_hybrid(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                             _ptr(signs), _ptr(cache), int(t_capacity), _ptr(v), _dtype_code(v),
                                             _ptr(seq_lens), int(max_len), _ptr(k_window), _dtype_code(k_window),
                                             int(k_window.shape[2]), _ptr(win_lens), float(scale), _ptr(out),
                                             _ptr(scores_out), _ptr(workspace),
                                             int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode_hybrid")


def octopus_vq_on_matrix_cores(cb, n_q_heads, n_kv_heads, n_q, v_bits, v_group):
    return bool(load().octopus_vq_on_matrix_cores(ctypes.byref(cb), int(n_q_heads), int(n_kv_heads), int(n_q),
                                                  int(v_bits), int(v_group)))


def octopus_probe_read(data, nontemporal, n_workgroups, sink, stream=None):
    """Measurement aid: plain streaming read of the device tensor `data` (uint8) by n_workgroups workgroups."""
    code = load().octopus_probe_read(_ptr(data), int(data.numel() * data.element_size()), int(bool(nontemporal)),
                                     int(n_workgroups), _ptr(sink), _stream_ptr(stream))
    _check(code, "octopus_probe_read")


def octopus_paged_pool_bytes(cb, n_pages, n_kv_heads):
    return int(load().octopus_paged_pool_bytes(ctypes.byref(cb), int(n_pages), int(n_kv_heads)))


def octopus_encode_paged(cb, keys, signs, k_pool, n_pages, block_table, start_pos=None, stream=None):
    """octopus_encode into a paged cache: k_pool device uint8 buffer of octopus_paged_pool_bytes(...) bytes,
    block_table device int32 [n_seq, max_pages_per_seq] contiguous."""
    assert keys.dim() == 4 and keys.stride(3) == 1 and block_table.is_contiguous()
    n_seq, n_new, n_kv, _ = keys.shape
    assert block_table.shape[0] == n_seq
    code = load().octopus_encode_paged(ctypes.byref(cb), _ptr(keys), _dtype_code(keys), keys.stride(0), keys.stride(1),
                                       keys.stride(2), n_seq, n_kv, n_new, _ptr(signs), _ptr(k_pool), int(n_pages),
                                       _ptr(block_table), int(block_table.shape[1]), _ptr(start_pos),
                                       _stream_ptr(stream))
    _check(code, "octopus_encode_paged")


def octopus_attn_decode_paged(cb, q, signs, k_pool, v_pool, block_table, seq_lens, max_len, scale, out, workspace,
                              stream=None):
    """octopus_attn_decode over a paged cache: v_pool device bf16 [n_pages, n_kv_heads, 64, d] contiguous."""
    assert q.is_contiguous() and v_pool.is_contiguous() and out.is_contiguous() and block_table.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_pages, n_kv = v_pool.shape[0], v_pool.shape[1]
    assert block_table.shape[0] == n_seq and v_pool.shape[2] == 64 and _dtype_code(v_pool) == DTYPE_BF16
    code = load().octopus_attn_decode_paged(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                            _ptr(signs), _ptr(k_pool), _ptr(v_pool), int(n_pages), _ptr(block_table),
                                            int(block_table.shape[1]), _ptr(seq_lens), int(max_len), float(scale),
                                            _ptr(out), _ptr(workspace),
                                            int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode_paged")


def octopus_attn_decode_paged_hybrid(cb, q, signs, k_pool, v_pool, block_table, seq_lens, max_len, k_window, win_lens,
                                     scale, out, workspace, stream=None):
    """octopus_attn_decode_paged plus a native-precision window: k_window device [n_seq, n_kv_heads, w_capacity, d]
    contiguous (fp32 or bf16), win_lens device int32 [n_seq]; the window's values follow the compressed tokens' in
    the sequence's value pages."""
    assert q.is_contiguous() and v_pool.is_contiguous() and out.is_contiguous() and block_table.is_contiguous()
    assert k_window.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_pages, n_kv = v_pool.shape[0], v_pool.shape[1]
    assert block_table.shape[0] == n_seq and v_pool.shape[2] == 64 and _dtype_code(v_pool) == DTYPE_BF16
    code = load().octopus_attn_decode_paged_hybrid(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                                   _ptr(signs), _ptr(k_pool), _ptr(v_pool), int(n_pages),
                                                   _ptr(block_table), int(block_table.shape[1]), _ptr(seq_lens),
                                                   int(max_len), _ptr(k_window), _dtype_code(k_window),
                                                   int(k_window.shape[2]), _ptr(win_lens), float(scale), _ptr(out),
                                                   _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                                   _stream_ptr(stream))
    _check(code, "octopus_attn_decode_paged_hybrid")


def octopus_encode_values_paged(v, bits, group, vq_pool, n_kv_heads, block_table, start_pos=None, stream=None):
    """octopus_encode_values into pages: v device [n_seq, n_new, n_kv_heads, d] (any strides, last one 1), vq_pool
    device uint8 of [n_pages][n_kv_heads][64] rows, block_table device int32 [n_seq, max_pages_per_seq]."""
    assert v.stride(-1) == 1 and block_table.is_contiguous()
    n_seq, n_new, n_kv, d = v.shape
    assert n_kv == n_kv_heads
    rb = octopus_vq_row_bytes(d, bits, group)
    n_pages = vq_pool.numel() * vq_pool.element_size() // (n_kv * 64 * rb)
    code = load().octopus_encode_values_paged(_ptr(v), _dtype_code(v), v.stride(0), v.stride(1), v.stride(2), n_seq, n_kv,
                                              n_new, d, int(bits), int(group), _ptr(vq_pool), int(n_pages),
                                              _ptr(block_table), int(block_table.shape[1]),
                                              _ptr(start_pos), _stream_ptr(stream))
    _check(code, "octopus_encode_values_paged")


def octopus_attn_decode_paged_vq(cb, q, signs, k_pool, vq_pool, v_bits, v_group, n_kv_heads, block_table, seq_lens,
                                 max_len, scale, out, workspace, stream=None):
    """octopus_attn_decode_paged over group-quantised value pages (vq_pool as octopus_encode_values_paged wrote it)."""
    assert q.is_contiguous() and out.is_contiguous() and block_table.is_contiguous()
    n_seq, n_q, n_qh, d = q.shape
    rb = octopus_vq_row_bytes(d, v_bits, v_group)
    n_pages = vq_pool.numel() * vq_pool.element_size() // (n_kv_heads * 64 * rb)
    assert block_table.shape[0] == n_seq
    code = load().octopus_attn_decode_paged_vq(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, int(n_kv_heads),
                                               n_q, _ptr(signs), _ptr(k_pool), _ptr(vq_pool), int(v_bits), int(v_group),
                                               int(n_pages), _ptr(block_table), int(block_table.shape[1]),
                                               _ptr(seq_lens), int(max_len), float(scale), _ptr(out), _ptr(workspace),
                                               int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode_paged_vq")


def octopus_encode_qjl_paged(cb, keys, signs, signs2, k_pool, qjl_pool, n_pages, block_table, start_pos=None,
                             stream=None):
    """octopus_encode_paged that also writes the QJL side-car into qjl_pool ([n_pages][n_kv_heads] side-car tiles)."""
    assert keys.stride(-1) == 1 and block_table.is_contiguous()
    n_seq, n_new, n_kv, _ = keys.shape
    code = load().octopus_encode_qjl_paged(ctypes.byref(cb), _ptr(keys), _dtype_code(keys), keys.stride(0),
                                           keys.stride(1), keys.stride(2), n_seq, n_kv, n_new, _ptr(signs), _ptr(signs2),
                                           _ptr(k_pool), _ptr(qjl_pool), int(n_pages), _ptr(block_table),
                                           int(block_table.shape[1]), _ptr(start_pos), _stream_ptr(stream))
    _check(code, "octopus_encode_qjl_paged")


def octopus_attn_decode_paged_qjl(cb, q, signs, signs2, k_pool, qjl_pool, v_pool, block_table, seq_lens, max_len, scale,
                                  out, workspace, stream=None):
    """octopus_attn_decode_paged with the QJL-corrected score; qjl_pool as octopus_encode_qjl_paged wrote it."""
    assert q.is_contiguous() and v_pool.is_contiguous() and out.is_contiguous() and block_table.is_contiguous()
    n_seq, n_q, n_qh, _ = q.shape
    n_pages, n_kv = v_pool.shape[0], v_pool.shape[1]
    assert block_table.shape[0] == n_seq and v_pool.shape[2] == 64 and _dtype_code(v_pool) == DTYPE_BF16
    code = load().octopus_attn_decode_paged_qjl(ctypes.byref(cb), _ptr(q), _dtype_code(q), n_seq, n_qh, n_kv, n_q,
                                                _ptr(signs), _ptr(signs2), _ptr(k_pool), _ptr(qjl_pool), _ptr(v_pool),
                                                int(n_pages), _ptr(block_table), int(block_table.shape[1]),
                                                _ptr(seq_lens), int(max_len), float(scale), _ptr(out), _ptr(workspace),
                                                int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    _check(code, "octopus_attn_decode_paged_qjl")


def octopus_profile_events(before, after):
    """before / after: torch.cuda.Event(enable_timing=True) that have been recorded once (so that their
    HIP handles exist), or None, None to cancel.  See include/octopus.h."""
    b = ctypes.c_void_p(before.cuda_event) if before is not None else ctypes.c_void_p(0)
    a = ctypes.c_void_p(after.cuda_event) if after is not None else ctypes.c_void_p(0)
    _check(load().octopus_profile_events(b, a), "octopus_profile_events")
