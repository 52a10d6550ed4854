/* Runs every entry point of the CPU oracle once on small seeded inputs.  Built by tests/test_sanitizers.py with
 * -fsanitize=address,undefined: an out-of-bounds access, a leak or undefined arithmetic ends it with a report. */
#include "../../oracle/octopus_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void) /* uniform in (-1, 1) */
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}

static void uniform_books(oracle_plan *p)
{
    for (int c = 0; c < p->n_class; ++c) {
        int K = 1 << p->b_dir[c], M = 1 << p->b_nrm[c];
        for (int k = 0; k < K; ++k) p->c_xi[c][k] = (double)(float)(-1.0 + (2.0 * k + 1.0) / K);
        for (int k = 0; k + 1 < K; ++k) p->b_xi[c][k] = 0.5 * (p->c_xi[c][k] + p->c_xi[c][k + 1]);
        for (int k = 0; k < M; ++k) p->c_rho[c][k] = (double)(float)(0.6 * (k + 0.5) / M);
        for (int k = 0; k + 1 < M; ++k) p->b_rho[c][k] = 0.5 * (p->c_rho[c][k] + p->c_rho[c][k + 1]);
    }
}

static int run_plan(oracle_plan *p, int n_keys, int n_q)
{
    int d = p->d, nt = p->n_tri, rb = oracle_record_bytes(p);
    double *keys = malloc(sizeof(double) * n_keys * d), *q = malloc(sizeof(double) * n_q * d);
    double *v = malloc(sizeof(double) * n_keys * d), *k_hat = malloc(sizeof(double) * n_keys * d);
    double *scores = malloc(sizeof(double) * n_q * n_keys), *out = malloc(sizeof(double) * n_q * d);
    int8_t *s = malloc(d), *s2 = malloc(d), *sigma = malloc((size_t)n_keys * d);
    double *gamma_r = malloc(sizeof(double) * n_keys);
    uint8_t *rec = malloc((size_t)n_keys * rb), *bad = malloc((size_t)n_keys * rb);
    for (int i = 0; i < n_keys * d; ++i) { keys[i] = 3.0 * rnd(); v[i] = rnd(); }
    for (int i = 0; i < d; ++i) keys[i] = 0.0;                 /* an all-zero key */
    for (int i = 0; i < d; ++i) keys[d + i] = (i == 5);        /* a one-hot key */
    for (int i = 0; i < n_q * d; ++i) q[i] = rnd();
    for (int i = 0; i < d; ++i) { s[i] = rnd() < 0 ? -1 : 1; s2[i] = rnd() < 0 ? -1 : 1; }
    int failures = 0;
    for (int mode = 0; mode < 5; ++mode) {
        if (mode == 2 && p->b_dir[0] > 4) continue;            /* the full grid at 5 bits is slow under a sanitizer */
        oracle_encode(p, keys, n_keys, s, mode, rec);
        int64_t c3[3] = { 0, 0, 0 }, c4[4] = { 0, 0, 0, 0 };
        oracle_classify_mode(p, keys, n_keys, s, mode, rec, 1e-6, c3);
        oracle_classify_both(p, keys, n_keys, s, mode, rec, 1e-6, c4);
        if (c3[0] != (int64_t)n_keys * nt || c4[0] != c3[0]) { printf("mode %d: own codes not all equal\n", mode); ++failures; }
    }
    oracle_encode(p, keys, n_keys, s, 1, rec);
    memcpy(bad, rec, (size_t)n_keys * rb);
    for (int t = 0; t < n_keys; ++t) bad[(size_t)t * rb + 4 + t % (rb - 4)] ^= (uint8_t)(1u << (t % 8));
    int64_t c4[4] = { 0, 0, 0, 0 };
    oracle_classify_both(p, keys, n_keys, s, 1, bad, 1e-6, c4);
    if (c4[0] + c4[1] + c4[2] + c4[3] != (int64_t)n_keys * nt) { printf("classification counts do not add up\n"); ++failures; }
    /* pack / unpack round trip */
    int32_t *idx = malloc(sizeof(int32_t) * 3 * nt);
    uint8_t *again = malloc(rb);
    for (int t = 0; t < n_keys; ++t) {
        double g;
        oracle_unpack_record(p, rec + (size_t)t * rb, &g, idx, idx + 2 * nt);
        oracle_pack_record(p, g, idx, idx + 2 * nt, again);
        if (memcmp(again, rec + (size_t)t * rb, rb) != 0) { printf("pack(unpack) differs at key %d\n", t); ++failures; break; }
    }
    oracle_reconstruct(p, rec, n_keys, s, k_hat);
    double gap = 0.0;
    oracle_attention(p, rec, n_keys, s, q, n_q, v, 1.0 / sqrt((double)d), scores, out, &gap);
    if (!(gap < 1e-9)) { printf("rotated and materialised scores differ by %g\n", gap); ++failures; }
    oracle_attention(p, rec, 0, s, q, n_q, v, 1.0, scores, out, &gap);   /* no keys at all */
    oracle_qjl_encode(p, keys, n_keys, s, s2, rec, sigma, gamma_r);
    oracle_attention_qjl(p, rec, n_keys, s, s2, sigma, gamma_r, q, n_q, v, 1.0 / sqrt((double)d), scores, out);
    for (int i = 0; i < n_q * d; ++i) if (!isfinite(out[i])) { printf("non-finite output\n"); ++failures; break; }
    free(keys); free(q); free(v); free(k_hat); free(scores); free(out); free(s); free(s2); free(sigma); free(gamma_r);
    free(rec); free(bad); free(idx); free(again);
    return failures;
}

int main(void)
{
    int failures = 0;
    oracle_plan a;
    memset(&a, 0, sizeof(a));
    a.d = 64; a.n_tri = 22; a.n_class = 1; a.class_ntri[0] = 22; a.b_dir[0] = 5; a.b_nrm[0] = 3;
    uniform_books(&a);
    failures += run_plan(&a, 70, 3);
    oracle_plan b;
    memset(&b, 0, sizeof(b));
    b.d = 128; b.n_tri = 43; b.n_class = 2; b.class_ntri[0] = 22; b.class_ntri[1] = 21;
    b.b_dir[0] = 4; b.b_nrm[0] = 2; b.b_dir[1] = 3; b.b_nrm[1] = 1;
    uniform_books(&b);
    failures += run_plan(&b, 40, 2);
    /* value codec: every bit width and group size, a constant group among them */
    for (int bits = 2; bits <= 4; ++bits)
        for (int g = 16; g <= 32; g += 16) {
            int d = 64, n = 9, rb = oracle_vq_row_bytes(d, bits, g);
            float *v = malloc(sizeof(float) * n * d);
            double *vh = malloc(sizeof(double) * n * d);
            uint8_t *rows = malloc((size_t)n * rb);
            for (int i = 0; i < n * d; ++i) v[i] = (float)rnd();
            for (int i = 0; i < g; ++i) v[i] = 0.25f;
            oracle_vq_encode(v, n, d, bits, g, rows);
            oracle_vq_decode(rows, n, d, bits, g, vh);
            for (int i = 0; i < n * d; ++i)
                if (!(fabs(vh[i] - (double)v[i]) <= 2.0 / ((1 << bits) - 1) * 0.5 + 1e-6)) { printf("value codec error too large\n"); ++failures; i = n * d; }
            free(v); free(vh); free(rows);
        }
    if (oracle_round_fp16(1.0) != 1.0) ++failures;
    printf(failures ? "FAILED (%d)\n" : "oracle driver ok\n", failures);
    return failures ? 1 : 0;
}
