"""OCTOPUS oracle: offline Lloyd-Max codebooks.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Follows Sec. 3.4 (Codebooks): two 1-D Lloyd-Max codebooks trained by the
alternating assignment / update iteration,
  C_rho(d, b_nrm) on [0, 1]  matched to the triplet-norm density Eq. (rho-pdf),
  C_xi(b_dir)     on [-1, 1] matched to the octahedral-coordinate marginal
                             Eq. (oct-marginal), shared by xi and eta,
with boundaries the midpoints of adjacent centroids (Alg. 1, Require).

Readings where the paper is silent:
  * the xi codebook is trained on the analytic Eq. (oct-marginal), the law of
    the samples the paper trains on, so the result is deterministic;
  * initial centroids are the equal-probability quantiles F^-1((k + 1/2) / L);
  * C_xi is symmetric (c_k = -c_{K-1-k}): the iteration runs on a = |xi| in
    [0, 1] with K/2 levels and is mirrored;
  * "to distortion 1e-10" is read as a floor on accuracy: the iteration runs
    to the fixed point (largest centroid move < 1e-13), which is below it;
  * centroids are rounded to fp32; boundaries are fp32(0.5 * (c_k + c_{k+1}))
    evaluated in fp64 on the fp32 centroids.

Cell integrals: rho uses the regularised incomplete beta function in x = r^2
(mass I_x(3/2, (d-3)/2); first moment B(2,(d-3)/2) / B(3/2,(d-3)/2) *
I_x(2, (d-3)/2)); xi uses Gauss-Legendre quadrature per cell (the density is
smooth on (0, 1)).
"""
from __future__ import annotations

import numpy as np
from scipy import special

_GL_X, _GL_W = np.polynomial.legendre.leggauss(64)


# ---- densities -------------------------------------------------------------

def f_rho(r, d):
    """Eq. (rho-pdf): density of a triplet norm for u uniform on S^{d-1}."""
    r = np.asarray(r, dtype=np.float64)
    return 2.0 * r * r * (1.0 - r * r) ** ((d - 5) / 2.0) / special.beta(1.5, (d - 3) / 2.0)


def f_xi(xi):
    """Eq. (oct-marginal): density of one octahedral coordinate on [-1, 1]."""
    a = np.abs(np.asarray(xi, dtype=np.float64))
    lead = 1.0 / (np.pi * np.sqrt(a * a + (1.0 - a) ** 2))
    return lead * ((1.0 - a) / (1.0 - 2.0 * a + 3.0 * a * a) + a / (2.0 - 4.0 * a + 3.0 * a * a))


def f_xi_integral_form(xi, n_nodes=200):
    """The integral form the closed form of Eq. (oct-marginal) is derived from
    (App., Octahedral Marginal): a second, independent evaluation."""
    a = abs(float(xi))
    x, w = np.polynomial.legendre.leggauss(n_nodes)

    def integ(lo, hi, fn):
        if hi <= lo:
            return 0.0
        s = 0.5 * (hi - lo) * x + 0.5 * (hi + lo)
        return float(np.sum(w * fn(s)) * 0.5 * (hi - lo))

    i1 = integ(0.0, 1.0 - a, lambda s: (a * a + s * s + (1.0 - a - s) ** 2) ** -1.5)
    i2 = integ(0.0, a, lambda s: (s * s + (1.0 - a) ** 2 + (s - a) ** 2) ** -1.5)
    return (i1 + i2) / (2.0 * np.pi)


# ---- cell mass / first moment ----------------------------------------------

def _rho_mass_moment(lo, hi, d):
    b2 = (d - 3) / 2.0
    mass = special.betainc(1.5, b2, hi * hi) - special.betainc(1.5, b2, lo * lo)
    ratio = special.beta(2.0, b2) / special.beta(1.5, b2)
    mom = ratio * (special.betainc(2.0, b2, hi * hi) - special.betainc(2.0, b2, lo * lo))
    return mass, mom


def _xi_half_mass_moment(lo, hi):
    """mass and first moment of a = |xi| (density 2 f_xi) on cells [lo, hi] in [0, 1]."""
    lo = np.asarray(lo, dtype=np.float64)[:, None]
    hi = np.asarray(hi, dtype=np.float64)[:, None]
    half = 0.5 * (hi - lo)
    s = half * _GL_X[None, :] + 0.5 * (hi + lo)
    dens = 2.0 * f_xi(s)
    mass = np.sum(_GL_W[None, :] * dens, axis=1) * half[:, 0]
    mom = np.sum(_GL_W[None, :] * dens * s, axis=1) * half[:, 0]
    return mass, mom


def _quantile(cdf, p, lo=0.0, hi=1.0):
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if cdf(mid) < p:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _lloyd(mass_moment, cdf, levels, lo, hi, tol=1e-13, max_iter=200000):
    """Alternating Lloyd-Max iteration on [lo, hi] from equal-probability quantiles."""
    c = np.array([_quantile(cdf, (k + 0.5) / levels, lo, hi) for k in range(levels)])
    for _ in range(max_iter):
        edges = np.concatenate(([lo], 0.5 * (c[:-1] + c[1:]), [hi]))
        mass, mom = mass_moment(edges[:-1], edges[1:])
        c_new = mom / mass
        move = np.max(np.abs(c_new - c))
        c = c_new
        if move < tol:
            break
    return c


def lloyd_max_rho_f64(d, b_nrm):
    levels = 1 << b_nrm
    b2 = (d - 3) / 2.0
    cdf = lambda r: special.betainc(1.5, b2, r * r)
    return _lloyd(lambda lo, hi: _rho_mass_moment(lo, hi, d), cdf, levels, 0.0, 1.0)


def lloyd_max_xi_f64(b_dir):
    levels = 1 << b_dir
    half = levels // 2

    def cdf(a):
        m, _ = _xi_half_mass_moment([0.0], [a])
        return float(m[0])

    pos = _lloyd(_xi_half_mass_moment, cdf, half, 0.0, 1.0)
    return np.concatenate((-pos[::-1], pos))


def _to_fp32_book(c64):
    c32 = np.asarray(c64, dtype=np.float64).astype(np.float32)
    mid = (0.5 * (c32[:-1].astype(np.float64) + c32[1:].astype(np.float64))).astype(np.float32)
    return c32, mid


def lloyd_max_rho(d, b_nrm):
    """(centroids, boundaries) as fp32 arrays."""
    return _to_fp32_book(lloyd_max_rho_f64(d, b_nrm))


def lloyd_max_xi(b_dir):
    return _to_fp32_book(lloyd_max_xi_f64(b_dir))


# ---- bit allocation ----------------------------------------------------------

def bit_split(b):
    """Sec. 3.3: the implemented (b+1, b-1) split for b in {2, 3, 4}; b = 1 is
    read as (1, 1) (Table rounding-ablation's b = 1 rows are only consistent
    with one bit per octahedral coordinate)."""
    b = int(b)
    if b == 1:
        return 1, 1
    if b in (2, 3, 4):
        return b + 1, b - 1
    raise ValueError(f"unsupported nominal bit width {b}")


def class_layout(d, bits):
    """Triplet classes for a nominal width: integer b -> one class; b + 1/2 ->
    the first ceil(n_tri / 2) triplets take the split of ceil(b), the rest
    the split of floor(b) (parity unpinned by the paper)."""
    n_tri = -(-d // 3)
    twice = int(round(2 * float(bits)))
    if abs(2 * float(bits) - twice) > 1e-9:
        raise ValueError("bits must be a multiple of 1/2")
    if twice % 2 == 0:
        bd, bn = bit_split(twice // 2)
        return n_tri, [(n_tri, bd, bn)]
    hi, lo = bit_split((twice + 1) // 2), bit_split((twice - 1) // 2)
    n0 = -(-n_tri // 2)
    return n_tri, [(n0, hi[0], hi[1]), (n_tri - n0, lo[0], lo[1])]
