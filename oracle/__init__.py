"""OCTOPUS CPU oracle (fp64).  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the HIP library never does and shares no code with it.

The arithmetic lives in octopus_oracle.c (codec, attention) and codebooks.py
(Lloyd-Max codebooks); this module only builds the C file with gcc, loads it
with ctypes and moves numpy arrays in and out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

from . import codebooks

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "octopus_oracle.c")
_LIB = os.path.join(_HERE, "liboctopus_oracle.so")
_MAXC = 64

MODE_SCALAR, MODE_LOCAL_3X3, MODE_FULL, MODE_INDEPENDENT, MODE_LOCAL_2X2 = 0, 1, 2, 3, 4


def build(force=False):
    """Compile the oracle's C file (gcc, -O2, OpenMP over keys)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _CPlan(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32),
        ("n_tri", ctypes.c_int32),
        ("n_class", ctypes.c_int32),
        ("class_ntri", ctypes.c_int32 * 2),
        ("b_dir", ctypes.c_int32 * 2),
        ("b_nrm", ctypes.c_int32 * 2),
        ("c_xi", (ctypes.c_double * _MAXC) * 2),
        ("b_xi", (ctypes.c_double * _MAXC) * 2),
        ("c_rho", (ctypes.c_double * _MAXC) * 2),
        ("b_rho", (ctypes.c_double * _MAXC) * 2),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.POINTER(_CPlan)
        vp = ctypes.c_void_p
        lib.oracle_stream_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.oracle_stream_bytes.restype = ctypes.c_int
        for name in ("oracle_dir_bytes", "oracle_nrm_bytes", "oracle_record_bytes"):
            getattr(lib, name).argtypes = [P]
            getattr(lib, name).restype = ctypes.c_int
        lib.oracle_hadamard.argtypes = [vp, vp, ctypes.c_int]
        lib.oracle_rotate.argtypes = [vp, vp, vp, ctypes.c_int]
        lib.oracle_rotate_inverse.argtypes = [vp, vp, vp, ctypes.c_int]
        lib.oracle_oct_encode.argtypes = [vp, vp, vp]
        lib.oracle_oct_decode.argtypes = [ctypes.c_double, ctypes.c_double, vp]
        lib.oracle_encode_key.argtypes = [P, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp, vp]
        lib.oracle_pack_record.argtypes = [P, ctypes.c_double, vp, vp, vp]
        lib.oracle_unpack_record.argtypes = [P, vp, vp, vp, vp]
        lib.oracle_encode.argtypes = [P, vp, ctypes.c_int64, vp, ctypes.c_int, vp]
        lib.oracle_reconstruct.argtypes = [P, vp, ctypes.c_int64, vp, vp]
        lib.oracle_attention.argtypes = [P, vp, ctypes.c_int64, vp, vp, ctypes.c_int, vp,
                                         ctypes.c_double, vp, vp, vp]
        lib.oracle_classify.argtypes = [P, vp, ctypes.c_int64, vp, vp, ctypes.c_double, vp]
        lib.oracle_classify_mode.argtypes = [P, vp, ctypes.c_int64, vp, ctypes.c_int, vp, ctypes.c_double, vp]
        lib.oracle_classify_both.argtypes = [P, vp, ctypes.c_int64, vp, ctypes.c_int, vp, ctypes.c_double, vp]
        lib.oracle_classify_both.restype = None
        lib.oracle_vq_row_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_vq_row_bytes.restype = ctypes.c_int
        lib.oracle_vq_encode.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
        lib.oracle_vq_encode.restype = None
        lib.oracle_vq_decode.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
        lib.oracle_vq_decode.restype = None
        lib.oracle_round_fp16.argtypes = [ctypes.c_double]
        lib.oracle_round_fp16.restype = ctypes.c_double
        lib.oracle_qjl_encode_key.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_qjl_encode_key.restype = None
        lib.oracle_qjl_encode.argtypes = [P, vp, ctypes.c_int64, vp, vp, vp, vp, vp]
        lib.oracle_qjl_encode.restype = None
        lib.oracle_qjl_estimate.argtypes = [vp, vp, vp, ctypes.c_double, ctypes.c_int]
        lib.oracle_qjl_estimate.restype = ctypes.c_double
        lib.oracle_attention_qjl.argtypes = [P, vp, ctypes.c_int64, vp, vp, vp, vp, vp, ctypes.c_int, vp,
                                             ctypes.c_double, vp, vp]
        lib.oracle_attention_qjl.restype = None
        for name in ("oracle_hadamard", "oracle_rotate", "oracle_rotate_inverse", "oracle_oct_encode",
                     "oracle_oct_decode", "oracle_encode_key", "oracle_pack_record",
                     "oracle_unpack_record", "oracle_encode", "oracle_reconstruct",
                     "oracle_attention", "oracle_classify"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


@dataclass
class Plan:
    """Codec parameters + fp32 codebooks (held as the fp64 values of the fp32 numbers)."""
    d: int
    n_tri: int
    classes: list  # [(ntri, b_dir, b_nrm), ...]
    c_xi: list = field(default_factory=list)   # per class, fp32 arrays
    b_xi: list = field(default_factory=list)
    c_rho: list = field(default_factory=list)
    b_rho: list = field(default_factory=list)

    def __post_init__(self):
        c = _CPlan()
        c.d, c.n_tri, c.n_class = self.d, self.n_tri, len(self.classes)
        for k, (nt, bd, bn) in enumerate(self.classes):
            c.class_ntri[k], c.b_dir[k], c.b_nrm[k] = nt, bd, bn
            for dst, src in ((c.c_xi, self.c_xi), (c.b_xi, self.b_xi), (c.c_rho, self.c_rho), (c.b_rho, self.b_rho)):
                for j, val in enumerate(np.asarray(src[k], dtype=np.float64)):
                    dst[k][j] = float(val)
        self._c = c

    @property
    def cptr(self):
        return ctypes.byref(self._c)

    @property
    def record_bytes(self):
        return _load().oracle_record_bytes(self.cptr)

    @property
    def dir_bytes(self):
        return _load().oracle_dir_bytes(self.cptr)

    @property
    def nrm_bytes(self):
        return _load().oracle_nrm_bytes(self.cptr)


_BOOK_CACHE = {}


def _xi_book(b_dir):
    key = ("xi", b_dir)
    if key not in _BOOK_CACHE:
        _BOOK_CACHE[key] = codebooks.lloyd_max_xi(b_dir)
    return _BOOK_CACHE[key]


def _rho_book(d, b_nrm):
    key = ("rho", d, b_nrm)
    if key not in _BOOK_CACHE:
        _BOOK_CACHE[key] = codebooks.lloyd_max_rho(d, b_nrm)
    return _BOOK_CACHE[key]


def make_plan_from_classes(d, classes, books=None):
    """classes = [(n_triplets, b_dir, b_nrm), ...]; books optionally overrides the
    codebooks with {(class index): (c_xi, b_xi, c_rho, b_rho)}."""
    n_tri = -(-d // 3)
    assert sum(c[0] for c in classes) == n_tri
    cx, bx, cr, br = [], [], [], []
    for k, (_, bd, bn) in enumerate(classes):
        if books is not None:
            a, b, c, e = books[k]
        else:
            a, b = _xi_book(bd)
            c, e = _rho_book(d, bn)
        cx.append(np.asarray(a, np.float32)); bx.append(np.asarray(b, np.float32))
        cr.append(np.asarray(c, np.float32)); br.append(np.asarray(e, np.float32))
    return Plan(d, n_tri, list(classes), cx, bx, cr, br)


def make_plan(d, bits):
    """Plan for a nominal bit width (Sec. 3.3 split; half-integers are two-class)."""
    n_tri, classes = codebooks.class_layout(d, bits)
    return make_plan_from_classes(d, classes)


def make_plan_pair(d, b_dir, b_nrm):
    """Single-class plan with an explicit (b_dir, b_nrm), as swept in App. D."""
    return make_plan_from_classes(d, [(-(-d // 3), b_dir, b_nrm)])


# ---- thin wrappers ------------------------------------------------------------

def stream_bytes(n, b):
    return _load().oracle_stream_bytes(int(n), int(b))


def hadamard(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_hadamard(_ptr(x), _ptr(y), x.shape[-1])
    return y


def signs_pm1(signs):
    s = np.ascontiguousarray(signs, dtype=np.int8)
    assert np.all(np.abs(s) == 1)
    return s


def rotate(x, signs):
    x, s = _f64(x), signs_pm1(signs)
    u = np.empty_like(x)
    _load().oracle_rotate(_ptr(x), _ptr(s), _ptr(u), x.shape[-1])
    return u


def rotate_inverse(u, signs):
    u, s = _f64(u), signs_pm1(signs)
    x = np.empty_like(u)
    _load().oracle_rotate_inverse(_ptr(u), _ptr(s), _ptr(x), u.shape[-1])
    return x


def oct_encode(t):
    t = _f64(t)
    xi, eta = ctypes.c_double(), ctypes.c_double()
    _load().oracle_oct_encode(_ptr(t), ctypes.byref(xi), ctypes.byref(eta))
    return xi.value, eta.value


def oct_decode(xi, eta):
    n = np.empty(3, dtype=np.float64)
    _load().oracle_oct_decode(float(xi), float(eta), _ptr(n))
    return n


def encode_key(plan, k, signs, mode=MODE_LOCAL_3X3):
    """One key -> dict(gamma, idx_dir, idx_nrm, u, xi_eta, s_star)."""
    k, s = _f64(k), signs_pm1(signs)
    nt = plan.n_tri
    gamma = ctypes.c_double()
    idx_dir = np.zeros(2 * nt, dtype=np.int32)
    idx_nrm = np.zeros(nt, dtype=np.int32)
    u = np.zeros(plan.d, dtype=np.float64)
    xe = np.zeros(2 * nt, dtype=np.float64)
    ss = np.zeros(nt, dtype=np.float64)
    _load().oracle_encode_key(plan.cptr, _ptr(k), _ptr(s), int(mode), ctypes.byref(gamma), _ptr(idx_dir),
                              _ptr(idx_nrm), _ptr(u), _ptr(xe), _ptr(ss))
    return dict(gamma=gamma.value, idx_dir=idx_dir, idx_nrm=idx_nrm, u=u, xi_eta=xe, s_star=ss)


def pack_record(plan, gamma, idx_dir, idx_nrm):
    rec = np.zeros(plan.record_bytes, dtype=np.uint8)
    a = np.ascontiguousarray(idx_dir, dtype=np.int32)
    b = np.ascontiguousarray(idx_nrm, dtype=np.int32)
    _load().oracle_pack_record(plan.cptr, float(gamma), _ptr(a), _ptr(b), _ptr(rec))
    return rec


def unpack_record(plan, rec):
    rec = np.ascontiguousarray(rec, dtype=np.uint8)
    gamma = ctypes.c_double()
    idx_dir = np.zeros(2 * plan.n_tri, dtype=np.int32)
    idx_nrm = np.zeros(plan.n_tri, dtype=np.int32)
    _load().oracle_unpack_record(plan.cptr, _ptr(rec), ctypes.byref(gamma), _ptr(idx_dir), _ptr(idx_nrm))
    return gamma.value, idx_dir, idx_nrm


def encode(plan, keys, signs, mode=MODE_LOCAL_3X3):
    """keys [n, d] -> canonical records [n, record_bytes] uint8."""
    keys, s = _f64(keys), signs_pm1(signs)
    assert keys.ndim == 2 and keys.shape[1] == plan.d
    rec = np.zeros((keys.shape[0], plan.record_bytes), dtype=np.uint8)
    _load().oracle_encode(plan.cptr, _ptr(keys), keys.shape[0], _ptr(s), int(mode), _ptr(rec))
    return rec


def reconstruct(plan, records, signs):
    """canonical records [n, record_bytes] -> reconstructed keys [n, d] (fp64)."""
    records, s = np.ascontiguousarray(records, dtype=np.uint8), signs_pm1(signs)
    out = np.zeros((records.shape[0], plan.d), dtype=np.float64)
    _load().oracle_reconstruct(plan.cptr, _ptr(records), records.shape[0], _ptr(s), _ptr(out))
    return out


def attention(plan, records, signs, q, v, scale):
    """q [n_q, d], v [n, d] -> (scores [n_q, n], out [n_q, d], form_gap)."""
    records, s = np.ascontiguousarray(records, dtype=np.uint8), signs_pm1(signs)
    q, v = _f64(np.atleast_2d(q)), _f64(v)
    n = records.shape[0]
    assert v.shape == (n, plan.d) and q.shape[1] == plan.d
    scores = np.zeros((q.shape[0], n), dtype=np.float64)
    out = np.zeros((q.shape[0], plan.d), dtype=np.float64)
    gap = ctypes.c_double()
    _load().oracle_attention(plan.cptr, _ptr(records), n, _ptr(s), _ptr(q), q.shape[0], _ptr(v), float(scale),
                             _ptr(scores), _ptr(out), ctypes.byref(gap))
    return scores, out, gap.value


def classify(plan, keys, signs, foreign_records, tol=1e-6, mode=MODE_LOCAL_3X3):
    """Per-triplet comparison of foreign records with Alg. 1 (in the given rounding mode):
    returns (n_equal, n_boundary_tie, n_hard)."""
    keys, s = _f64(keys), signs_pm1(signs)
    fr = np.ascontiguousarray(foreign_records, dtype=np.uint8)
    assert fr.shape == (keys.shape[0], plan.record_bytes)
    counts = np.zeros(3, dtype=np.int64)
    _load().oracle_classify_mode(plan.cptr, _ptr(keys), keys.shape[0], _ptr(s), int(mode), _ptr(fr), float(tol),
                                 _ptr(counts))
    return int(counts[0]), int(counts[1]), int(counts[2])


def classify_both(plan, keys, signs, foreign_records, tol=1e-6, mode=MODE_LOCAL_3X3):
    """The same comparison under both readings of "within tol": returns (n_equal, n_tie_literal, n_tie_scaled_only,
    n_hard).  Literal: tol on every compared quantity (xi, eta and p_z included).  Scaled: the tolerance on the
    octahedral coordinates is tol / min(l1, 1), a triplet with l1 < tol admits any direction (what classify()
    applies).  n_tie_scaled_only counts the triplets only the scaled reading admits."""
    keys, s = _f64(keys), signs_pm1(signs)
    fr = np.ascontiguousarray(foreign_records, dtype=np.uint8)
    assert fr.shape == (keys.shape[0], plan.record_bytes)
    counts = np.zeros(4, dtype=np.int64)
    _load().oracle_classify_both(plan.cptr, _ptr(keys), keys.shape[0], _ptr(s), int(mode), _ptr(fr), float(tol),
                                 _ptr(counts))
    return tuple(int(c) for c in counts)


# ---- optional 1-bit QJL residual (Sec. 3.6) -------------------------------------------------------

def round_fp16(x):
    return _load().oracle_round_fp16(float(x))


def qjl_encode(plan, keys, signs, signs2, records):
    """keys [n, d], canonical records [n, record_bytes] -> (sigma [n, d] int8 of +-1, gamma_r [n] fp16 values)."""
    keys, s, s2 = _f64(keys), signs_pm1(signs), signs_pm1(signs2)
    rec = np.ascontiguousarray(records, dtype=np.uint8)
    n = keys.shape[0]
    assert rec.shape == (n, plan.record_bytes)
    sigma = np.zeros((n, plan.d), dtype=np.int8)
    gamma_r = np.zeros(n, dtype=np.float64)
    _load().oracle_qjl_encode(plan.cptr, _ptr(keys), n, _ptr(s), _ptr(s2), _ptr(rec), _ptr(sigma), _ptr(gamma_r))
    return sigma, gamma_r


def qjl_residual(plan, k, signs, signs2, idx_dir, idx_nrm):
    """One key -> (sigma [d], gamma_r, r [d]) from explicit codes."""
    k, s, s2 = _f64(k), signs_pm1(signs), signs_pm1(signs2)
    a = np.ascontiguousarray(idx_dir, dtype=np.int32)
    b = np.ascontiguousarray(idx_nrm, dtype=np.int32)
    sigma = np.zeros(plan.d, dtype=np.int8)
    r = np.zeros(plan.d, dtype=np.float64)
    g = ctypes.c_double()
    _load().oracle_qjl_encode_key(plan.cptr, _ptr(k), _ptr(s), _ptr(s2), _ptr(a), _ptr(b), _ptr(sigma), ctypes.byref(g),
                                  _ptr(r))
    return sigma, g.value, r


def qjl_estimate(q_rot, signs2, sigma, gamma_r):
    q_rot, s2 = _f64(q_rot), signs_pm1(signs2)
    sg = np.ascontiguousarray(sigma, dtype=np.int8)
    return _load().oracle_qjl_estimate(_ptr(q_rot), _ptr(s2), _ptr(sg), float(gamma_r), int(q_rot.shape[0]))


def attention_qjl(plan, records, signs, signs2, sigma, gamma_r, q, v, scale):
    """-> (scores [n_q, n], out [n_q, d]) with scores scale * (q . k^ + gamma * estimate)."""
    records, s, s2 = np.ascontiguousarray(records, dtype=np.uint8), signs_pm1(signs), signs_pm1(signs2)
    q, v = _f64(np.atleast_2d(q)), _f64(v)
    n = records.shape[0]
    sg = np.ascontiguousarray(sigma, dtype=np.int8)
    gr = _f64(gamma_r)
    assert sg.shape == (n, plan.d) and gr.shape == (n,) and v.shape == (n, plan.d)
    scores = np.zeros((q.shape[0], n), dtype=np.float64)
    out = np.zeros((q.shape[0], plan.d), dtype=np.float64)
    _load().oracle_attention_qjl(plan.cptr, _ptr(records), n, _ptr(s), _ptr(s2), _ptr(sg), _ptr(gr), _ptr(q), q.shape[0],
                                 _ptr(v), float(scale), _ptr(scores), _ptr(out))
    return scores, out


# ---- value codec: per-group uniform quantisation (Sec. 4; parity unpinned by the paper) ----------------

def vq_row_bytes(d, bits, group):
    return int(_load().oracle_vq_row_bytes(int(d), int(bits), int(group)))


def vq_encode(v, bits, group):
    """v [n, d] (fp32 values) -> rows uint8 [n, vq_row_bytes]"""
    v = np.ascontiguousarray(v, dtype=np.float32)
    n, d = v.shape
    assert d % group == 0 and group % 8 == 0
    rows = np.zeros((n, vq_row_bytes(d, bits, group)), dtype=np.uint8)
    _load().oracle_vq_encode(_ptr(v), n, d, int(bits), int(group), _ptr(rows))
    return rows


def vq_decode(rows, d, bits, group):
    """rows uint8 [n, vq_row_bytes] -> v^ float64 [n, d]"""
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    assert rows.shape[1] == vq_row_bytes(d, bits, group)
    out = np.zeros((rows.shape[0], d), dtype=np.float64)
    _load().oracle_vq_decode(_ptr(rows), rows.shape[0], d, int(bits), int(group), _ptr(out))
    return out


# ---- hybrid cache: compressed tokens followed by a native-precision window (Sec. 4, default recipe) ----

def attention_hybrid(plan, records, signs, k_window, q, v, scale):
    """Attention over n compressed tokens (canonical records) followed by w tokens whose keys are kept at
    native precision (k_window [w, d]); v [n + w, d].  Written as the definition: the key matrix is the
    reconstructed keys stacked on the window's keys, then softmax(scale * q K^T) V.
    -> (scores [n_q, n + w], out [n_q, d])."""
    q, v, kw = _f64(np.atleast_2d(q)), _f64(v), _f64(k_window).reshape(-1, plan.d)
    k_all = np.concatenate([reconstruct(plan, records, signs), kw], axis=0)
    assert v.shape == k_all.shape
    scores = scale * (q @ k_all.T)
    out = np.zeros((q.shape[0], plan.d))
    if k_all.shape[0]:
        w = np.exp(scores - scores.max(axis=1, keepdims=True))
        out = (w / w.sum(axis=1, keepdims=True)) @ v
    return scores, out
