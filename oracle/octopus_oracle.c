/*
 * OCTOPUS CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 implementation of the OCTOPUS key codec and of
 * attention over the reconstructed keys, written from the paper so that a
 * reader can check it against the paper by eye.  It shares nothing with the
 * HIP library (no headers, tables, helpers).  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may load it.
 *
 * What follows what:
 *   rotation            Eq. (rotation), Sec. 3.1: u = H diag(s) u~, H the
 *                       normalised Sylvester Hadamard matrix, written out as
 *                       the O(d^2) matrix product (no butterfly).
 *   triplets            Sec. 3.2: ceil(d/3) contiguous triplets, zero padded.
 *   Oct / Oct^-1        Eq. (oct-encode), Eq. (oct-decode), sign(0) = +1.
 *   encoder             Alg. 1 (encoder with joint rounding), step by step.
 *   stream packing      Alg. 1 last step; stream sizes are the ones the KV
 *                       ratios of Table (kernel speed) imply.
 *   scores, attention   Eq. (score-exact), Alg. 2: computed here as the plain
 *                       definition softmax(scale * q K^T) V on the
 *                       materialised reconstructed keys k^ = gamma R^T u^.
 *   QJL side-car        Sec. 3.6 "1-bit QJL residual" and App. "QJL Residual
 *                       Estimator": sign sketch of the rotated-frame residual
 *                       under a second sign-flipped Hadamard rotation, residual
 *                       norm rounded to fp16, corrected score.
 *
 *   value codec         Sec. 4 ("value-side group size in {16, 32}") and the
 *                       "value dequantization" step of Alg. 2's description.
 *                       The paper gives the group size and (through the KV
 *                       ratios of Table (kernel speed)) the size, b d / 8
 *                       code bytes + 8 bytes per group, and nothing else: the
 *                       codec here is uniform asymmetric min/max quantisation
 *                       per group with an fp32 scale and an fp32 zero point.
 *                       PARITY UNPINNED by the paper beyond the byte count.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   eps = 1e-20 for both clamped divisors; searchsorted counts boundaries
 *   strictly below the value; candidate order dx outer, dy inner, each
 *   -1,0,+1, strict '>' keeps the first maximum; streams are LSB-first;
 *   index counts are padded with zeros to whole byte groups.
 *
 * Parity unpinned by the paper (fixed by this build's readings only): the
 * two-class plans for half-integer bit widths, eps, tie order, bit order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OCT_EPS 1e-20
#define OCT_MAXC 64

typedef struct {
    int32_t d;             /* head dimension, power of two                    */
    int32_t n_tri;         /* ceil(d / 3)                                     */
    int32_t n_class;       /* 1, or 2 for a half-integer nominal bit width    */
    int32_t class_ntri[2]; /* class 0 = first class_ntri[0] triplets          */
    int32_t b_dir[2];      /* bits per octahedral coordinate, per class       */
    int32_t b_nrm[2];      /* bits per triplet norm, per class                */
    double c_xi[2][OCT_MAXC];  /* C_xi centroids, ascending                   */
    double b_xi[2][OCT_MAXC];  /* B_xi midpoints (2^b_dir - 1 used)           */
    double c_rho[2][OCT_MAXC]; /* C_rho centroids, ascending                  */
    double b_rho[2][OCT_MAXC]; /* B_rho midpoints (2^b_nrm - 1 used)          */
} oracle_plan;

/* ---- stream geometry (Table kernel-speed KV ratios) ---------------------- */

static int gcd_int(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

/* bytes of a stream of n indices of b bits: the index count is padded to a
 * whole number of byte groups, a group being the fewest indices that fill
 * whole bytes. */
int oracle_stream_bytes(int n, int b)
{
    if (b <= 0 || n <= 0) return 0;
    int g = 8 / gcd_int(b, 8);
    int groups = (n + g - 1) / g;
    return groups * (g * b / 8);
}

int oracle_dir_bytes(const oracle_plan *p)
{
    int s = 0;
    for (int c = 0; c < p->n_class; ++c) s += oracle_stream_bytes(2 * p->class_ntri[c], p->b_dir[c]);
    return s;
}

int oracle_nrm_bytes(const oracle_plan *p)
{
    int s = 0;
    for (int c = 0; c < p->n_class; ++c) s += oracle_stream_bytes(p->class_ntri[c], p->b_nrm[c]);
    return s;
}

/* canonical record of one key: [gamma fp32][dir streams][nrm streams] */
int oracle_record_bytes(const oracle_plan *p) { return 4 + oracle_dir_bytes(p) + oracle_nrm_bytes(p); }

static int class_of(const oracle_plan *p, int i) { return (i < p->class_ntri[0]) ? 0 : 1; }

/* ---- rotation: Eq. (rotation) ------------------------------------------- */

/* y = H x with H[i][j] = (-1)^popcount(i & j) / sqrt(d), the definition. */
void oracle_hadamard(const double *x, double *y, int d)
{
    double inv = 1.0 / sqrt((double)d);
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int j = 0; j < d; ++j)
            acc += (__builtin_parity((unsigned)(i & j)) ? -x[j] : x[j]);
        y[i] = acc * inv;
    }
}

/* u = R x = H (s . x) */
void oracle_rotate(const double *x, const int8_t *s, double *u, int d)
{
    double *t = (double *)malloc(sizeof(double) * d);
    for (int j = 0; j < d; ++j) t[j] = (double)s[j] * x[j];
    oracle_hadamard(t, u, d);
    free(t);
}

/* x = R^T u = s . (H u) */
void oracle_rotate_inverse(const double *u, const int8_t *s, double *x, int d)
{
    oracle_hadamard(u, x, d);
    for (int j = 0; j < d; ++j) x[j] *= (double)s[j];
}

/* ---- octahedral map: Eq. (oct-encode), Eq. (oct-decode) ------------------ */

static double sgn1(double v) { return (v >= 0.0) ? 1.0 : -1.0; } /* sign(0) = +1 */

void oracle_oct_encode(const double t[3], double *xi, double *eta)
{
    double l1 = fabs(t[0]) + fabs(t[1]) + fabs(t[2]);
    double den = (l1 > OCT_EPS) ? l1 : OCT_EPS;
    double px = t[0] / den, py = t[1] / den, pz = t[2] / den;
    if (pz >= 0.0) { *xi = px; *eta = py; }
    else { *xi = sgn1(px) * (1.0 - fabs(py)); *eta = sgn1(py) * (1.0 - fabs(px)); }
}

void oracle_oct_decode(double xi, double eta, double n[3])
{
    double r = 1.0 - fabs(xi) - fabs(eta);
    double a = xi, b = eta;
    if (r < 0.0) { a = sgn1(xi) * (1.0 - fabs(eta)); b = sgn1(eta) * (1.0 - fabs(xi)); }
    double nn = sqrt(a * a + b * b + r * r);
    n[0] = a / nn; n[1] = b / nn; n[2] = r / nn;
}

/* searchsorted: number of boundaries strictly below v */
static int count_below(const double *bnd, int n, double v)
{
    int j = 0;
    for (int k = 0; k < n; ++k) if (bnd[k] < v) ++j;
    return j;
}

static double clip01(double v) { return v < 0.0 ? 0.0 : (v > 1.0 ? 1.0 : v); }
static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* ---- encoder: Alg. 1 ----------------------------------------------------- */

/* The encoder is put together from four parts, each of which can be read against the paper on its own:
 *   unit_rotated      gamma = ||k||, u = H (s . k / gamma), zero-padded to whole triplets (Alg. 1, first steps);
 *   the seed          per axis, the centroid cell the octahedral coordinate falls into (searchsorted on B_xi);
 *   a candidate set   which cells around the seed compete: a list of (dx, dy) offsets per rounding mode, in
 *                     the order they are tried (App. E; Sec. 3.5 for the default), or the whole K x K grid;
 *   the choice        the candidate whose direction has the largest cosine with the triplet, the first one on
 *                     ties; the norm code is then the cell of that cosine (of the triplet's own length for the
 *                     independent rounds) in B_rho.
 * Rounding modes: 0 = the seed alone, 1 = the seed's 3x3 neighbourhood (default), 2 = the full grid,
 * 3 = three independent nearest-centroid rounds (Sec. 3.5, first paragraph: the radius code is the centroid
 * nearest to rho_i itself; the "scalar" rows of the rounding ablation), 4 = local 2x2 (App. E names it without
 * defining it; read as the seed cell and its upper neighbour per axis, clamped at the rim: this window
 * reproduces the printed local 2x2 rows, whereas the two centroids that bracket the coordinate reproduce the
 * 3x3 rows instead). */

typedef struct { int8_t dx, dy; } cell_offset;

static const cell_offset kSeedOnly[] = {{0, 0}};
static const cell_offset kNeighbours3x3[] = {{-1, -1}, {-1, 0}, {-1, 1}, {0, -1}, {0, 0}, {0, 1}, {1, -1}, {1, 0}, {1, 1}};
static const cell_offset kUpper2x2[] = {{0, 0}, {0, 1}, {1, 0}, {1, 1}};

typedef struct {
    int cell_x, cell_y;   /* centroid indices of the chosen direction */
    double cosine;        /* t . n^ of the chosen direction (-inf: nothing tried yet) */
} direction_choice;

/* gamma and the rotated unit key, zero-padded to 3 * n_tri coordinates (u must hold that many). */
static double unit_rotated(const oracle_plan *p, const double *key, const int8_t *signs, double *u)
{
    const int d = p->d;
    double *scaled = (double *)malloc(sizeof(double) * (size_t)d);
    double sq = 0.0;
    for (int j = 0; j < d; ++j) sq += key[j] * key[j];
    const double gamma = sqrt(sq);
    const double divisor = (gamma > OCT_EPS) ? gamma : OCT_EPS;
    for (int j = 0; j < d; ++j) scaled[j] = key[j] / divisor;
    for (int j = d; j < 3 * p->n_tri; ++j) u[j] = 0.0;
    oracle_rotate(scaled, signs, u, d);
    free(scaled);
    return gamma;
}

/* t . Oct^-1(C[ix], C[iy]) */
static double cell_cosine(const double t[3], const double *centroids, int ix, int iy)
{
    double n[3];
    oracle_oct_decode(centroids[ix], centroids[iy], n);
    return t[0] * n[0] + t[1] * n[1] + t[2] * n[2];
}

/* Offers one cell to the running choice; a later cell wins only if strictly better. */
static void offer_cell(direction_choice *best, const double t[3], const double *centroids, int ix, int iy)
{
    const double c = cell_cosine(t, centroids, ix, iy);
    if (c > best->cosine) {
        best->cosine = c;
        best->cell_x = ix;
        best->cell_y = iy;
    }
}

static direction_choice choose_direction(const double t[3], const double *centroids, int n_levels, int seed_x,
                                         int seed_y, int mode)
{
    direction_choice best = {seed_x, seed_y, -INFINITY};
    if (mode == 2) {
        for (int ix = 0; ix < n_levels; ++ix)
            for (int iy = 0; iy < n_levels; ++iy) offer_cell(&best, t, centroids, ix, iy);
        return best;
    }
    const cell_offset *window = kSeedOnly;
    int n_cells = 1;
    if (mode == 1) { window = kNeighbours3x3; n_cells = 9; }
    if (mode == 4) { window = kUpper2x2; n_cells = 4; }
    for (int c = 0; c < n_cells; ++c)
        offer_cell(&best, t, centroids, clampi(seed_x + window[c].dx, 0, n_levels - 1),
                   clampi(seed_y + window[c].dy, 0, n_levels - 1));
    return best;
}

/* Outputs per key: gamma, idx_dir[2*n_tri] (order (i,0),(i,1)), idx_nrm[n_tri];
 * optional diagnostics (may be NULL): u[d], xi_eta[2*n_tri], s_star[n_tri] (the chosen cosine). */
void oracle_encode_key(const oracle_plan *p, const double *k, const int8_t *s, int mode,
                       double *gamma_out, int32_t *idx_dir, int32_t *idx_nrm,
                       double *u_out, double *xi_eta_out, double *s_star_out)
{
    double *u = (double *)malloc(sizeof(double) * (size_t)(3 * p->n_tri));
    *gamma_out = unit_rotated(p, k, s, u);
    if (u_out) memcpy(u_out, u, sizeof(double) * p->d);

    for (int i = 0; i < p->n_tri; ++i) {
        const int cls = class_of(p, i);
        const int n_dir = 1 << p->b_dir[cls], n_nrm = 1 << p->b_nrm[cls];
        const double *t = u + 3 * i;
        double xi, eta;
        oracle_oct_encode(t, &xi, &eta);
        const int seed_x = count_below(p->b_xi[cls], n_dir - 1, xi);
        const int seed_y = count_below(p->b_xi[cls], n_dir - 1, eta);
        const direction_choice best = choose_direction(t, p->c_xi[cls], n_dir, seed_x, seed_y, mode);
        idx_dir[2 * i] = best.cell_x;
        idx_dir[2 * i + 1] = best.cell_y;
        const double radial = (mode == 3) ? sqrt(t[0] * t[0] + t[1] * t[1] + t[2] * t[2]) : best.cosine;
        idx_nrm[i] = count_below(p->b_rho[cls], n_nrm - 1, clip01(radial));
        if (xi_eta_out) { xi_eta_out[2 * i] = xi; xi_eta_out[2 * i + 1] = eta; }
        if (s_star_out) s_star_out[i] = best.cosine;
    }
    free(u);
}

/* ---- bit streams --------------------------------------------------------- */

static void put_bits(uint8_t *stream, int64_t bitpos, int nbits, uint32_t v)
{
    for (int b = 0; b < nbits; ++b, ++bitpos)
        if ((v >> b) & 1u) stream[bitpos >> 3] |= (uint8_t)(1u << (bitpos & 7));
}

static uint32_t get_bits(const uint8_t *stream, int64_t bitpos, int nbits)
{
    uint32_t v = 0;
    for (int b = 0; b < nbits; ++b, ++bitpos)
        v |= (uint32_t)((stream[bitpos >> 3] >> (bitpos & 7)) & 1u) << b;
    return v;
}

/* record = [gamma as fp32, little endian][dir c0][dir c1][nrm c0][nrm c1] */
void oracle_pack_record(const oracle_plan *p, double gamma, const int32_t *idx_dir,
                        const int32_t *idx_nrm, uint8_t *rec)
{
    memset(rec, 0, (size_t)oracle_record_bytes(p));
    float g = (float)gamma;
    memcpy(rec, &g, 4);
    uint8_t *dir = rec + 4;
    int t0 = 0;
    for (int c = 0; c < p->n_class; ++c) {
        for (int i = 0; i < p->class_ntri[c]; ++i) {
            put_bits(dir, (int64_t)(2 * i) * p->b_dir[c], p->b_dir[c], (uint32_t)idx_dir[2 * (t0 + i)]);
            put_bits(dir, (int64_t)(2 * i + 1) * p->b_dir[c], p->b_dir[c], (uint32_t)idx_dir[2 * (t0 + i) + 1]);
        }
        dir += oracle_stream_bytes(2 * p->class_ntri[c], p->b_dir[c]);
        t0 += p->class_ntri[c];
    }
    uint8_t *nrm = dir;
    t0 = 0;
    for (int c = 0; c < p->n_class; ++c) {
        for (int i = 0; i < p->class_ntri[c]; ++i)
            put_bits(nrm, (int64_t)i * p->b_nrm[c], p->b_nrm[c], (uint32_t)idx_nrm[t0 + i]);
        nrm += oracle_stream_bytes(p->class_ntri[c], p->b_nrm[c]);
        t0 += p->class_ntri[c];
    }
}

void oracle_unpack_record(const oracle_plan *p, const uint8_t *rec, double *gamma,
                          int32_t *idx_dir, int32_t *idx_nrm)
{
    float g;
    memcpy(&g, rec, 4);
    *gamma = (double)g;
    const uint8_t *dir = rec + 4;
    int t0 = 0;
    for (int c = 0; c < p->n_class; ++c) {
        for (int i = 0; i < p->class_ntri[c]; ++i) {
            idx_dir[2 * (t0 + i)] = (int32_t)get_bits(dir, (int64_t)(2 * i) * p->b_dir[c], p->b_dir[c]);
            idx_dir[2 * (t0 + i) + 1] = (int32_t)get_bits(dir, (int64_t)(2 * i + 1) * p->b_dir[c], p->b_dir[c]);
        }
        dir += oracle_stream_bytes(2 * p->class_ntri[c], p->b_dir[c]);
        t0 += p->class_ntri[c];
    }
    const uint8_t *nrm = dir;
    t0 = 0;
    for (int c = 0; c < p->n_class; ++c) {
        for (int i = 0; i < p->class_ntri[c]; ++i)
            idx_nrm[t0 + i] = (int32_t)get_bits(nrm, (int64_t)i * p->b_nrm[c], p->b_nrm[c]);
        nrm += oracle_stream_bytes(p->class_ntri[c], p->b_nrm[c]);
        t0 += p->class_ntri[c];
    }
}

/* encode n_keys keys (row-major [n_keys][d]) to canonical records */
void oracle_encode(const oracle_plan *p, const double *keys, int64_t n_keys, const int8_t *s,
                   int mode, uint8_t *records)
{
    int rb = oracle_record_bytes(p);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 3 * p->n_tri);
        double gamma;
        oracle_encode_key(p, keys + t * p->d, s, mode, &gamma, idx, idx + 2 * p->n_tri, NULL, NULL, NULL);
        oracle_pack_record(p, gamma, idx, idx + 2 * p->n_tri, records + t * rb);
        free(idx);
    }
}

/* ---- decoder ------------------------------------------------------------- */

/* rotated-frame reconstruction u^ (length 3*n_tri, caller uses first d) */
void oracle_decode_rotated(const oracle_plan *p, const int32_t *idx_dir, const int32_t *idx_nrm,
                           double *u_hat)
{
    for (int i = 0; i < p->n_tri; ++i) {
        int c = class_of(p, i);
        double n[3];
        oracle_oct_decode(p->c_xi[c][idx_dir[2 * i]], p->c_xi[c][idx_dir[2 * i + 1]], n);
        double rho = p->c_rho[c][idx_nrm[i]];
        u_hat[3 * i] = rho * n[0];
        u_hat[3 * i + 1] = rho * n[1];
        u_hat[3 * i + 2] = rho * n[2];
    }
}

/* materialised k^ = gamma * R^T u^ for n_keys records; coordinates >= d of the
 * last triplet are dropped */
void oracle_reconstruct(const oracle_plan *p, const uint8_t *records, int64_t n_keys,
                        const int8_t *s, double *k_hat)
{
    int rb = oracle_record_bytes(p), d = p->d;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 3 * p->n_tri);
        double *uh = (double *)malloc(sizeof(double) * 3 * p->n_tri);
        double gamma;
        oracle_unpack_record(p, records + t * rb, &gamma, idx, idx + 2 * p->n_tri);
        oracle_decode_rotated(p, idx, idx + 2 * p->n_tri, uh);
        oracle_rotate_inverse(uh, s, k_hat + t * d, d);
        for (int j = 0; j < d; ++j) k_hat[t * d + j] *= gamma;
        free(idx);
        free(uh);
    }
}

/* Attention of n_q queries (sharing one KV head) over the first n_keys
 * records: scores[qi][t] = scale * q_qi . k^_t, p = softmax_t, out = p V.
 * Also evaluates the rotated-frame form gamma * (R q) . u^ of Eq.
 * (score-exact) and returns the largest absolute difference between the two
 * forms in *form_gap (the oracle's self check of Prop. invariance). */
void oracle_attention(const oracle_plan *p, const uint8_t *records, int64_t n_keys,
                      const int8_t *s, const double *q, int n_q, const double *v, double scale,
                      double *scores, double *out, double *form_gap)
{
    int d = p->d, rb = oracle_record_bytes(p);
    double *q_rot = (double *)malloc(sizeof(double) * (size_t)n_q * d);
    for (int qi = 0; qi < n_q; ++qi) oracle_rotate(q + (size_t)qi * d, s, q_rot + (size_t)qi * d, d);
    double gap = 0.0;
#pragma omp parallel for schedule(static) reduction(max : gap)
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 3 * p->n_tri);
        double *uh = (double *)malloc(sizeof(double) * 3 * p->n_tri);
        double *kh = (double *)malloc(sizeof(double) * d);
        double gamma;
        oracle_unpack_record(p, records + t * rb, &gamma, idx, idx + 2 * p->n_tri);
        oracle_decode_rotated(p, idx, idx + 2 * p->n_tri, uh);
        oracle_rotate_inverse(uh, s, kh, d);
        for (int qi = 0; qi < n_q; ++qi) {
            double direct = 0.0, rotated = 0.0;
            for (int j = 0; j < d; ++j) {
                direct += q[(size_t)qi * d + j] * (gamma * kh[j]);
                rotated += q_rot[(size_t)qi * d + j] * uh[j];
            }
            rotated *= gamma;
            double g = fabs(direct - rotated);
            if (g > gap) gap = g;
            scores[(size_t)qi * n_keys + t] = scale * direct;
        }
        free(idx);
        free(uh);
        free(kh);
    }
    if (form_gap) *form_gap = gap;
    for (int qi = 0; qi < n_q; ++qi) {
        const double *sc = scores + (size_t)qi * n_keys;
        double *o = out + (size_t)qi * d;
        for (int j = 0; j < d; ++j) o[j] = 0.0;
        if (n_keys == 0) continue;
        double m = -INFINITY;
        for (int64_t t = 0; t < n_keys; ++t) if (sc[t] > m) m = sc[t];
        double l = 0.0;
        for (int64_t t = 0; t < n_keys; ++t) {
            double w = exp(sc[t] - m);
            l += w;
            for (int j = 0; j < d; ++j) o[j] += w * v[t * d + j];
        }
        for (int j = 0; j < d; ++j) o[j] /= l;
    }
    free(q_rot);
}

/* ---- optional 1-bit QJL residual (Sec. 3.6) ------------------------------ */

/* Nearest binary16 value (ties to even), returned as a double; values beyond
 * the fp16 range saturate to the largest finite fp16. */
double oracle_round_fp16(double x)
{
    if (x == 0.0 || x != x) return x;
    double a = fabs(x);
    if (a >= 65520.0) return (x < 0 ? -65504.0 : 65504.0);
    int e;
    frexp(a, &e);                 /* a = m * 2^e, m in [0.5, 1) */
    int ulp_exp = e - 11;         /* 11 significant bits for normal numbers */
    if (ulp_exp < -24) ulp_exp = -24; /* subnormal spacing 2^-24 */
    double ulp = ldexp(1.0, ulp_exp);
    double r = nearbyint(a / ulp) * ulp; /* default rounding mode: ties to even */
    return x < 0 ? -r : r;
}

/* Side-car of one key from its codes: r = u - u^ in the rotated frame (u the
 * rotated unit key, u^ the reconstruction the codes define, d coordinates),
 * sigma = sign(H diag(s2) r) with sign(0) = +1, gamma_r = fp16(||r||_2).
 * sigma_out[j] in {+1, -1}. */
void oracle_qjl_encode_key(const oracle_plan *p, const double *k, const int8_t *s, const int8_t *s2,
                           const int32_t *idx_dir, const int32_t *idx_nrm, int8_t *sigma_out,
                           double *gamma_r_out, double *r_out)
{
    int d = p->d;
    double *buf = (double *)calloc((size_t)3 * p->n_tri + 3 * d, sizeof(double));
    double *uh = buf, *ku = buf + 3 * p->n_tri, *u = ku + d, *y = u + d;
    double g2 = 0.0;
    for (int j = 0; j < d; ++j) g2 += k[j] * k[j];
    double gamma = sqrt(g2);
    double den = (gamma > OCT_EPS) ? gamma : OCT_EPS;
    for (int j = 0; j < d; ++j) ku[j] = k[j] / den;
    oracle_rotate(ku, s, u, d);
    oracle_decode_rotated(p, idx_dir, idx_nrm, uh);
    double n2 = 0.0;
    for (int j = 0; j < d; ++j) { ku[j] = u[j] - uh[j]; n2 += ku[j] * ku[j]; }   /* ku now holds r */
    if (r_out) memcpy(r_out, ku, sizeof(double) * d);
    oracle_rotate(ku, s2, y, d);
    for (int j = 0; j < d; ++j) sigma_out[j] = (y[j] >= 0.0) ? 1 : -1;
    *gamma_r_out = oracle_round_fp16(sqrt(n2));
    free(buf);
}

/* Side-cars of n_keys keys whose codes are in `records` (canonical layout). */
void oracle_qjl_encode(const oracle_plan *p, const double *keys, int64_t n_keys, const int8_t *s,
                       const int8_t *s2, const uint8_t *records, int8_t *sigma, double *gamma_r)
{
    int rb = oracle_record_bytes(p), d = p->d;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 3 * p->n_tri);
        double gamma;
        oracle_unpack_record(p, records + t * rb, &gamma, idx, idx + 2 * p->n_tri);
        oracle_qjl_encode_key(p, keys + t * d, s, s2, idx, idx + 2 * p->n_tri, sigma + t * d, gamma_r + t, NULL);
        free(idx);
    }
}

/* QJL estimate of q_rot . r:  sqrt(pi / (2 d)) * gamma_r * (H diag(s2) q_rot) . sigma */
double oracle_qjl_estimate(const double *q_rot, const int8_t *s2, const int8_t *sigma, double gamma_r, int d)
{
    double *y = (double *)malloc(sizeof(double) * d);
    oracle_rotate(q_rot, s2, y, d);
    double acc = 0.0;
    for (int j = 0; j < d; ++j) acc += y[j] * (double)sigma[j];
    free(y);
    return sqrt(M_PI / (2.0 * d)) * gamma_r * acc;
}

/* Attention with corrected scores: scale * (q . k^_t + gamma_t * estimate_t).
 * sigma: [n_keys][d] of +-1, gamma_r: [n_keys]. */
void oracle_attention_qjl(const oracle_plan *p, const uint8_t *records, int64_t n_keys, const int8_t *s,
                          const int8_t *s2, const int8_t *sigma, const double *gamma_r, const double *q,
                          int n_q, const double *v, double scale, double *scores, double *out)
{
    int d = p->d, rb = oracle_record_bytes(p);
    double *q_rot = (double *)malloc(sizeof(double) * (size_t)n_q * d);
    for (int qi = 0; qi < n_q; ++qi) oracle_rotate(q + (size_t)qi * d, s, q_rot + (size_t)qi * d, d);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 3 * p->n_tri);
        double *uh = (double *)malloc(sizeof(double) * 3 * p->n_tri);
        double *kh = (double *)malloc(sizeof(double) * d);
        double gamma;
        oracle_unpack_record(p, records + t * rb, &gamma, idx, idx + 2 * p->n_tri);
        oracle_decode_rotated(p, idx, idx + 2 * p->n_tri, uh);
        oracle_rotate_inverse(uh, s, kh, d);
        for (int qi = 0; qi < n_q; ++qi) {
            double direct = 0.0;
            for (int j = 0; j < d; ++j) direct += q[(size_t)qi * d + j] * (gamma * kh[j]);
            double est = oracle_qjl_estimate(q_rot + (size_t)qi * d, s2, sigma + t * d, gamma_r[t], d);
            scores[(size_t)qi * n_keys + t] = scale * (direct + gamma * est);
        }
        free(idx);
        free(uh);
        free(kh);
    }
    for (int qi = 0; qi < n_q; ++qi) {
        const double *sc = scores + (size_t)qi * n_keys;
        double *o = out + (size_t)qi * d;
        for (int j = 0; j < d; ++j) o[j] = 0.0;
        if (n_keys == 0) continue;
        double m = -INFINITY;
        for (int64_t t = 0; t < n_keys; ++t) if (sc[t] > m) m = sc[t];
        double l = 0.0;
        for (int64_t t = 0; t < n_keys; ++t) {
            double w = exp(sc[t] - m);
            l += w;
            for (int j = 0; j < d; ++j) o[j] += w * v[t * d + j];
        }
        for (int j = 0; j < d; ++j) o[j] /= l;
    }
    free(q_rot);
}

/* ---- classification of a foreign record against Alg. 1 ------------------- */

/* For one key and a record produced elsewhere, decide per triplet whether the
 * foreign codes are (0) the oracle's, (1) what Alg. 1 yields if every
 * comparison whose two sides lie within tol of each other may go either way
 * (a decision-boundary tie), or (2) neither.  counts[0..2] are incremented.
 * Comparisons covered: the sign tests of Eq. (oct-encode) (p_z >= 0 and, on
 * the folded branch, sign(p_x), sign(p_y)), xi / eta against B_xi, the
 * candidate argmax (any window candidate within tol of the window maximum),
 * clip(s) against B_rho.
 * tol is a distance in the coordinates of the rotated unit key u, the quantity
 * every decision of Alg. 1 derives from.  Scores and clip(s) are in those
 * units; the octahedral coordinates are not: p = t / l1, so a coordinate
 * change of tol moves p_x, p_y, p_z, xi and eta by about tol / l1.  Their
 * comparisons therefore use tol_p = tol / min(l1, 1), and a triplet whose l1
 * is itself below tol (numerically zero, its direction rounding noise) admits
 * every sign pattern and every seed. */
static int window_admits(const oracle_plan *p, int c, const double t[3], double xi, double eta,
                         int fx, int fy, int fn, double tol, double tol_p, int mode)
{
    int K = 1 << p->b_dir[c], M = 1 << p->b_nrm[c];
    const double *cx = p->c_xi[c], *bx = p->b_xi[c];
    double n[3];
    oracle_oct_decode(cx[fx], cx[fy], n);
    double sf = t[0] * n[0] + t[1] * n[1] + t[2] * n[2];
    int jx_lo = count_below(bx, K - 1, xi - tol_p), jx_hi = count_below(bx, K - 1, xi + tol_p);
    int jy_lo = count_below(bx, K - 1, eta - tol_p), jy_hi = count_below(bx, K - 1, eta + tol_p);
    /* the radius code: from clip(s*) of the chosen direction, in mode 3 from rho_i itself */
    double radial = (mode == 3) ? sqrt(t[0] * t[0] + t[1] * t[1] + t[2] * t[2]) : sf;
    double cs = clip01(radial);
    int n_lo = count_below(p->b_rho[c], M - 1, cs - tol), n_hi = count_below(p->b_rho[c], M - 1, cs + tol);
    if (fn < n_lo || fn > n_hi) return 0;
    if (mode == 2) { /* full grid: the seeds play no part */
        double best = -INFINITY;
        for (int ax = 0; ax < K; ++ax)
            for (int ay = 0; ay < K; ++ay) {
                oracle_oct_decode(cx[ax], cx[ay], n);
                double sc = t[0] * n[0] + t[1] * n[1] + t[2] * n[2];
                if (sc > best) best = sc;
            }
        return sf >= best - tol;
    }
    int r = (mode == 0 || mode == 3) ? 0 : 1;
    for (int jx = jx_lo; jx <= jx_hi; ++jx)
        for (int jy = jy_lo; jy <= jy_hi; ++jy) {
            int in_window = 0;
            double best = -INFINITY;
            for (int dx = -r; dx <= r; ++dx)
                for (int dy = -r; dy <= r; ++dy) {
                    if (mode == 4 && (dx < 0 || dy < 0)) continue;
                    int ax = clampi(jx + dx, 0, K - 1), ay = clampi(jy + dy, 0, K - 1);
                    oracle_oct_decode(cx[ax], cx[ay], n);
                    double sc = t[0] * n[0] + t[1] * n[1] + t[2] * n[2];
                    if (sc > best) best = sc;
                    if (ax == fx && ay == fy) in_window = 1;
                }
            if (in_window && sf >= best - tol) return 1;
        }
    return 0;
}

/* literal != 0: the plain reading of "within tol" -- the same tol on every compared quantity, the octahedral
 * coordinates included (tol_p = tol), and no exemption for a numerically zero triplet.  literal == 0: tol_p
 * scaled by 1 / l1 as described above.  Every tie under the literal rule is one under the scaled rule. */
static void classify_key(const oracle_plan *p, const double *k, const int8_t *s, int mode, int literal,
                         const uint8_t *foreign, double tol, int64_t counts[3])
{
    int nt = p->n_tri;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * 6 * nt);
    int32_t *o_dir = idx, *o_nrm = idx + 2 * nt, *f_dir = idx + 3 * nt, *f_nrm = idx + 5 * nt;
    double *u = (double *)calloc((size_t)3 * nt + p->d, sizeof(double));
    double gamma, fg;
    oracle_encode_key(p, k, s, mode, &gamma, o_dir, o_nrm, u, NULL, NULL);
    oracle_unpack_record(p, foreign, &fg, f_dir, f_nrm);
    for (int i = 0; i < nt; ++i) {
        if (o_dir[2 * i] == f_dir[2 * i] && o_dir[2 * i + 1] == f_dir[2 * i + 1] && o_nrm[i] == f_nrm[i]) {
            counts[0]++;
            continue;
        }
        int c = class_of(p, i);
        int K = 1 << p->b_dir[c], M = 1 << p->b_nrm[c];
        const double *t = u + 3 * i; /* u: d rotated coordinates, then zero padding */
        int fx = f_dir[2 * i], fy = f_dir[2 * i + 1], fn = f_nrm[i];
        int ok = 0;
        if (fx < K && fy < K && fn < M) {
            double l1 = fabs(t[0]) + fabs(t[1]) + fabs(t[2]);
            double den = (l1 > OCT_EPS) ? l1 : OCT_EPS;
            double px = t[0] / den, py = t[1] / den, pz = t[2] / den;
            double tol_p = literal ? tol : ((l1 > tol) ? tol / (l1 < 1.0 ? l1 : 1.0) : 4.0);
            if (pz >= -tol_p) ok = window_admits(p, c, t, px, py, fx, fy, fn, tol, tol_p, mode); /* unfolded branch */
            if (!ok && pz < tol_p)                                                     /* folded branch */
                for (int vx = 0; vx < 2 && !ok; ++vx)
                    for (int vy = 0; vy < 2 && !ok; ++vy) {
                        double sx = vx ? 1.0 : -1.0, sy = vy ? 1.0 : -1.0;
                        if (fabs(px) > tol_p && sx != sgn1(px)) continue;
                        if (fabs(py) > tol_p && sy != sgn1(py)) continue;
                        ok = window_admits(p, c, t, sx * (1.0 - fabs(py)), sy * (1.0 - fabs(px)), fx, fy, fn, tol,
                                           tol_p, mode);
                    }
        }
        counts[ok ? 1 : 2]++;
    }
    free(idx);
    free(u);
}

void oracle_classify_key_mode(const oracle_plan *p, const double *k, const int8_t *s, int mode,
                              const uint8_t *foreign, double tol, int64_t counts[3])
{
    classify_key(p, k, s, mode, 0, foreign, tol, counts);
}

/* Both rules at once: counts4 = { equal, ties under the literal rule, ties only the scaled rule admits, hard }. */
void oracle_classify_both(const oracle_plan *p, const double *keys, int64_t n_keys, const int8_t *s, int mode,
                          const uint8_t *foreign_records, double tol, int64_t counts4[4])
{
    int rb = oracle_record_bytes(p);
    int64_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma omp parallel for schedule(static) reduction(+ : c0, c1, c2, c3)
    for (int64_t t = 0; t < n_keys; ++t) {
        int64_t lit[3] = { 0, 0, 0 }, sca[3] = { 0, 0, 0 };
        classify_key(p, keys + t * p->d, s, mode, 1, foreign_records + t * rb, tol, lit);
        if (lit[1] + lit[2] == 0) { c0 += lit[0]; continue; }
        classify_key(p, keys + t * p->d, s, mode, 0, foreign_records + t * rb, tol, sca);
        c0 += lit[0]; c1 += lit[1]; c2 += sca[1] - lit[1]; c3 += sca[2];
    }
    counts4[0] += c0; counts4[1] += c1; counts4[2] += c2; counts4[3] += c3;
}

void oracle_classify_key(const oracle_plan *p, const double *k, const int8_t *s,
                         const uint8_t *foreign, double tol, int64_t counts[3])
{
    oracle_classify_key_mode(p, k, s, 1, foreign, tol, counts);
}

void oracle_classify_mode(const oracle_plan *p, const double *keys, int64_t n_keys, const int8_t *s, int mode,
                          const uint8_t *foreign_records, double tol, int64_t counts[3])
{
    int rb = oracle_record_bytes(p);
    int64_t c0 = 0, c1 = 0, c2 = 0;
#pragma omp parallel for schedule(static) reduction(+ : c0, c1, c2)
    for (int64_t t = 0; t < n_keys; ++t) {
        int64_t c[3] = { 0, 0, 0 };
        oracle_classify_key_mode(p, keys + t * p->d, s, mode, foreign_records + t * rb, tol, c);
        c0 += c[0]; c1 += c[1]; c2 += c[2];
    }
    counts[0] += c0; counts[1] += c1; counts[2] += c2;
}

void oracle_classify(const oracle_plan *p, const double *keys, int64_t n_keys, const int8_t *s,
                     const uint8_t *foreign_records, double tol, int64_t counts[3])
{
    int rb = oracle_record_bytes(p);
    int64_t c0 = 0, c1 = 0, c2 = 0;
#pragma omp parallel for schedule(static) reduction(+ : c0, c1, c2)
    for (int64_t t = 0; t < n_keys; ++t) {
        int64_t c[3] = { 0, 0, 0 };
        oracle_classify_key(p, keys + t * p->d, s, foreign_records + t * rb, tol, c);
        c0 += c[0]; c1 += c[1]; c2 += c[2];
    }
    counts[0] += c0; counts[1] += c1; counts[2] += c2;
}

/* ---- value codec: per-group uniform quantisation ------------------------- */

/* The paper fixes the group size g in {16, 32}, the bit width b (that of the
 * keys) and, through the printed KV ratios, the size b d / 8 + 8 d / g bytes
 * per value row.  Everything else is this build's reading (parity unpinned by
 * the paper): per group of g consecutive channels
 *     lo = min v, hi = max v, scale = (hi - lo) / (2^b - 1), zero = lo,
 *     code_j = clamp(rint((v_j - lo) / scale), 0, 2^b - 1)   (0 if scale = 0),
 *     v^_j = zero + scale * code_j,
 * scale and zero stored as fp32.  The integer decision (rint, ties to even) is
 * taken in fp32, the precision of the stored metadata and of the kernel: every
 * operation below is a single correctly rounded fp32 operation, so that an
 * IEEE fp32 implementation reproduces the codes bit for bit.
 * Row layout: [codes, channel j at bit b j, LSB first][per group: scale, zero]. */
int oracle_vq_row_bytes(int d, int b, int g) { return b * d / 8 + (d / g) * 8; }

void oracle_vq_encode(const float *v, int64_t n, int d, int b, int g, uint8_t *rows)
{
    int rb = oracle_vq_row_bytes(d, b, g), levels = (1 << b) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        uint8_t *row = rows + t * rb;
        memset(row, 0, (size_t)rb);
        for (int grp = 0; grp < d / g; ++grp) {
            const float *x = v + t * d + grp * g;
            float lo = x[0], hi = x[0];
            for (int j = 1; j < g; ++j) {
                if (x[j] < lo) lo = x[j];
                if (x[j] > hi) hi = x[j];
            }
            volatile float range = hi - lo;               /* volatile: one rounding per operation */
            volatile float scale = range / (float)levels;
            for (int j = 0; j < g; ++j) {
                uint32_t code = 0;
                if (scale > 0.0f) {
                    volatile float off = x[j] - lo;
                    volatile float r = off / scale;
                    float c = nearbyintf(r);              /* default rounding mode: ties to even */
                    if (c < 0.0f) c = 0.0f;
                    if (c > (float)levels) c = (float)levels;
                    code = (uint32_t)c;
                }
                put_bits(row, (int64_t)b * (grp * g + j), b, code);
            }
            float meta[2] = { scale, lo };
            memcpy(row + b * d / 8 + grp * 8, meta, 8);
        }
    }
}

void oracle_vq_decode(const uint8_t *rows, int64_t n, int d, int b, int g, double *v_hat)
{
    int rb = oracle_vq_row_bytes(d, b, g);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const uint8_t *row = rows + t * rb;
        for (int j = 0; j < d; ++j) {
            float meta[2];
            memcpy(meta, row + b * d / 8 + (j / g) * 8, 8);
            v_hat[t * d + j] = (double)meta[1] + (double)meta[0] * (double)get_bits(row, (int64_t)b * j, b);
        }
    }
}
