/*
 * octopus.h -- C ABI of the MI355X (gfx950) implementation of the OCTOPUS key
 * codec and of fused decode attention over the compressed keys.
 *
 * The three operations are the ones the paper's problem statement names:
 *   octopus_build_codebooks   Sec. 3.3 (bit split) + Sec. 3.4 (codebooks)
 *   octopus_encode            Alg. 1 (encoder with joint rounding), Sec. 3.1-3.5
 *   octopus_attn_decode       Alg. 2 (split-K flash decode), Eq. (score-exact)
 * Further entry points, each documented where it is declared below:
 *   octopus_encode_rounding   the encoder's rounding variants (App. E)
 *   octopus_encode_qjl, octopus_attn_decode_qjl    the 1-bit QJL residual (Sec. 3.6)
 *   octopus_encode_values, octopus_attn_decode_vq  group-quantised values (Sec. 4, Alg. 2)
 *   octopus_attn_decode_hybrid                     native-precision window (Sec. 4)
 *   octopus_encode_paged, octopus_attn_decode_paged, octopus_attn_decode_paged_hybrid,
 *   octopus_encode_values_paged, octopus_attn_decode_paged_vq,
 *   octopus_encode_qjl_paged, octopus_attn_decode_paged_qjl
 *                                                  the same codec and attention over a paged cache
 *
 * Conventions
 *   - Plain C.  Every function returns 0 (OCTOPUS_OK) or a negative error
 *     code; nothing throws.  octopus_strerror() names a code.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP
 *     device memory owned by the caller (e.g. the storage of a torch tensor).
 *     The library never allocates or frees device memory, never copies
 *     between host and device, and never synchronises: every launch goes to
 *     the caller's stream (`stream` is a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns once the work is enqueued.
 *   - Arguments are validated on the host before anything is launched; a
 *     call that returns an error has launched nothing.
 *   - All multi-byte values are little endian.
 *
 * Compressed cache layout (device)
 *   One region per (sequence, KV head), regions ordered [n_seq][n_kv_heads],
 *   each holding t_capacity tokens, t_capacity a multiple of 64.  A key's
 *   canonical record is the byte string of Alg. 1's return value,
 *       [gamma: fp32][dir stream: dir_bytes][nrm stream: nrm_bytes]
 *   (LSB-first packing, index n of a b-bit stream at bits [n*b, (n+1)*b);
 *   direction indices ordered (i,0),(i,1); index counts padded with zero
 *   indices to whole byte groups; two-class plans store
 *   [dir class0][dir class1][nrm class0][nrm class1]),
 *   zero-padded to plan.granules * 16 bytes.  Records are interleaved in
 *   tiles of 64 tokens so that a wavefront with one key per lane loads 16
 *   bytes per lane fully coalesced: byte x of the record of token t is at
 *       region + ((t/64 * granules + x/16) * 64 + t%64) * 16 + x%16 .
 *   octopus_cache_bytes() gives the size of the whole cache.
 */
#ifndef OCTOPUS_H_
#define OCTOPUS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OCTOPUS_OK            0
#define OCTOPUS_EINVAL       (-1) /* null pointer, negative size, inconsistent shapes          */
#define OCTOPUS_EUNSUPPORTED (-2) /* head_dim / bit width / dtype / head ratio not built in    */
#define OCTOPUS_EWORKSPACE   (-3) /* workspace missing, misaligned or too small                */
#define OCTOPUS_EHIP         (-4) /* the HIP runtime refused a launch                          */
#define OCTOPUS_ESCRATCH     (-5) /* shapes exceed the static scratch of octopus_attn_decode_static */

#define OCTOPUS_DTYPE_F32  0
#define OCTOPUS_DTYPE_BF16 1

#define OCTOPUS_MAX_LEVELS 64
#define OCTOPUS_TILE       64     /* tokens per cache tile */

/* Pure function of (head_dim, bits): Sec. 3.2 (triplets), Sec. 3.3 (split). */
typedef struct octopus_plan {
    int32_t head_dim;       /* d: 64, 128 or 256                                              */
    int32_t n_tri;          /* ceil(d / 3) coordinate triplets, the last zero padded          */
    int32_t n_class;        /* 1 for integer nominal bits, 2 for b + 1/2                      */
    int32_t class_ntri[2];  /* class 0 = first class_ntri[0] triplets, class 1 = the rest     */
    int32_t b_dir[2];       /* bits per octahedral coordinate (xi and eta each)               */
    int32_t b_nrm[2];       /* bits per triplet norm                                          */
    int32_t dir_bytes;      /* size of the direction stream(s) of one key                     */
    int32_t nrm_bytes;      /* size of the norm stream(s) of one key                          */
    int32_t record_bytes;   /* 4 + dir_bytes + nrm_bytes: canonical record                    */
    int32_t granules;       /* ceil(record_bytes / 16): 16-byte units per key on the device   */
} octopus_plan_t;

/* Codebooks of Sec. 3.4: ascending fp32 centroids and the midpoints of
 * adjacent centroids (Alg. 1, Require), per class.  Caller-owned host POD. */
typedef struct octopus_codebooks {
    octopus_plan_t plan;
    float c_xi[2][OCTOPUS_MAX_LEVELS];   /* 2^b_dir centroids on [-1, 1], c[k] = -c[K-1-k]     */
    float b_xi[2][OCTOPUS_MAX_LEVELS];   /* 2^b_dir - 1 boundaries                             */
    float c_rho[2][OCTOPUS_MAX_LEVELS];  /* 2^b_nrm centroids on [0, 1]                        */
    float b_rho[2][OCTOPUS_MAX_LEVELS];  /* 2^b_nrm - 1 boundaries                             */
} octopus_codebooks_t;

/* Sec. 3.3 + Sec. 3.4.  Host only, deterministic, no device work.
 * bits: nominal bits per coordinate b in {1, 1.5, 2, 2.5, 3, 4}.  Integer b
 * uses the implemented split (b_dir, b_nrm) = (b+1, b-1) for b = 2, 3, 4 and
 * (1, 1) for b = 1; b + 1/2 gives the first ceil(n_tri/2) triplets the split
 * of b + 1 and the rest the split of b.  C_rho is the Lloyd-Max quantiser of
 * Eq. (rho-pdf), C_xi that of Eq. (oct-marginal), both iterated to their
 * fixed point from equal-probability quantiles.
 * head_dim: 64, 128 or 256.  out: host, caller-owned, fully overwritten.
 * Errors: EINVAL (out NULL), EUNSUPPORTED (head_dim or bits not listed). */
int octopus_build_codebooks(int32_t head_dim, float bits, octopus_codebooks_t *out);

/* Same with an explicit single-class (b_dir, b_nrm), 1 <= b_dir, b_nrm <= 6: the
 * bit-allocation sweep of App. D.  Codebooks are built for every such pair.  Kernels:
 * the pairs that are a built bit width ((1,1), (3,1), (4,2), (5,3)) have every kernel;
 * at head_dim 128 the other pairs of the App. D table -- (1,3), (2,2), (1,5), (2,4),
 * (3,3), (5,1), (2,6), (3,5), (4,4), (6,2) -- have octopus_encode and octopus_attn_decode
 * (and its _static / _hybrid forms) over bf16 values without score output and with fewer
 * than 32 query rows per KV head; every other call with them, and every other pair,
 * answers EUNSUPPORTED. */
int octopus_build_codebooks_pair(int32_t head_dim, int32_t b_dir, int32_t b_nrm, octopus_codebooks_t *out);

/* Bytes of a compressed cache of n_seq x n_kv_heads regions of t_capacity
 * tokens (0 if an argument is invalid: t_capacity not a positive multiple of
 * 64, counts < 1, cb NULL). */
size_t octopus_cache_bytes(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_kv_heads, int64_t t_capacity);

/* Alg. 1 with the local 3x3 candidate set, for n_new new tokens of every
 * (sequence, KV head).
 *   cb          host.  Codebooks (only c_* are read; boundaries are recomputed
 *               as midpoints).
 *   keys        device, element (s, t, h, c) at keys[s*stride_seq + t*stride_tok
 *               + h*stride_head + c], t in [0, n_new), c in [0, d) contiguous;
 *               strides in elements, multiples of 8 (rows are read 16 bytes
 *               at a time); base 16-byte aligned.
 *   key_dtype   OCTOPUS_DTYPE_F32 or OCTOPUS_DTYPE_BF16.
 *   signs       device, [n_kv_heads][d/8] bytes: bit j%8 of byte j/8 set means
 *               s_j = -1 (Eq. (rotation): one sign vector per head).
 *   cache       device, 16-byte aligned, layout above; token t of sequence s is
 *               written to slot start_pos[s] + t.  Other slots are untouched.
 *   start_pos   device [n_seq] int32 >= 0 (a negative entry is read as 0), or NULL
 *               for all zeros.  Slots beyond t_capacity are not written (the
 *               caller must size the cache).
 * Errors: EINVAL (also n_seq or n_kv_heads above 65535), EUNSUPPORTED (plan /
 * dtype without a kernel; centroids not ascending, two boundaries of C_xi closer than 1 / (4 * 2^b_dir), which the
 * kernel's seed search does not resolve, or C_xi not antisymmetric (c_xi[K - 1 - k] == -c_xi[k] exactly, as the
 * Lloyd-Max codebook of the symmetric marginal is: the kernel keeps one quadrant of the direction table) --
 * never the case for the codebooks octopus_build_codebooks returns), EHIP. */
int octopus_encode(const octopus_codebooks_t *cb,
                   const void *keys, int32_t key_dtype,
                   int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                   int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                   const uint8_t *signs,
                   void *cache, int64_t t_capacity,
                   const int32_t *start_pos,
                   void *stream);

/* ---- encoder rounding variants (App. E, "Rounding ablation") ----
 * Encoder-only: the bitstream and the decoder are those of octopus_encode.
 *   SEED         Alg. 1 with the candidate window {(0,0)}: the direction codes are the
 *                scalar seeds, the norm code comes from clip(s) of that direction.
 *   LOCAL_3X3    Alg. 1 as printed (what octopus_encode does).
 *   FULL         all 2^b_dir x 2^b_dir direction candidates.
 *   INDEPENDENT  three independent nearest-centroid rounds (Sec. 3.5, first paragraph):
 *                seeds for the direction, the centroid nearest to rho_i for the norm.
 *   LOCAL_2X2    the seed cell and its upper neighbour per axis (4 candidates).
 * Candidates are visited first index outer, second inner, ascending; the first maximum wins. */
#define OCTOPUS_ROUND_SEED        0
#define OCTOPUS_ROUND_LOCAL_3X3   1
#define OCTOPUS_ROUND_FULL        2
#define OCTOPUS_ROUND_INDEPENDENT 3
#define OCTOPUS_ROUND_LOCAL_2X2   4

/* octopus_encode with the rounding mode `rounding` (OCTOPUS_ROUND_*); EINVAL for another
 * value.  Other arguments and errors as octopus_encode. */
int octopus_encode_rounding(const octopus_codebooks_t *cb,
                            const void *keys, int32_t key_dtype,
                            int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                            int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                            const uint8_t *signs,
                            void *cache, int64_t t_capacity,
                            const int32_t *start_pos,
                            int32_t rounding,
                            void *stream);

/* ---- optional 1-bit QJL residual (Sec. 3.6, "OCTOPUS-QJL") ----
 * Side-car of a key: sigma = sign(H diag(s') r) for the residual r = u - u^ of
 * the rotated unit key (d bits) and gamma_r = ||r||_2 as fp16.  Device layout,
 * one region per (sequence, KV head) ordered like the cache, per tile of 64
 * tokens: [d/32 words][64 tokens] uint32 (bit j%32 of word j/32 set when
 * sigma_j = -1; sign(0) = +1), then [64 tokens] fp16 gamma_r:
 * 64 * (d/8 + 2) bytes per tile. */

/* Bytes of the side-car buffer (0 if an argument is invalid). */
size_t octopus_qjl_bytes(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_kv_heads, int64_t t_capacity);

/* octopus_encode that also writes the side-car of every encoded token.
 *   signs2      device, [n_kv_heads][d/8] bytes like signs: the sign vector s'
 *               of the second rotation, drawn independently of s.
 *   qjl         device, 4-byte aligned, octopus_qjl_bytes(...) bytes; slots of
 *               other tokens are untouched.
 * Other arguments and errors as octopus_encode; EINVAL if signs2 or qjl is NULL. */
int octopus_encode_qjl(const octopus_codebooks_t *cb,
                       const void *keys, int32_t key_dtype,
                       int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                       int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                       const uint8_t *signs, const uint8_t *signs2,
                       void *cache, void *qjl, int64_t t_capacity,
                       const int32_t *start_pos,
                       void *stream);

/* Bytes of device workspace octopus_attn_decode needs for these shapes
 * (rotated queries + split-K partials); 0 if an argument is invalid. */
size_t octopus_attn_decode_workspace(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_q_heads,
                                     int32_t n_kv_heads, int32_t n_q, int64_t max_len);

/* Alg. 2 + the split merge: out = softmax_t(scale * q . k^_t) V over the
 * tokens t < seq_lens[s] of each sequence, with k^ the key the codes define
 * (Eq. (score-exact)); the uncompressed key is never written to memory.
 * Every query of a sequence sees all seq_lens[s] tokens (no causal mask).
 *   q           device, [n_seq][n_q][n_q_heads][d] contiguous, q_dtype F32/BF16.
 *               Query head h uses KV head h / (n_q_heads / n_kv_heads).
 *   signs       device, as for octopus_encode.
 *   cache       device, as written by octopus_encode with the same cb.
 *   v           device, [n_seq][n_kv_heads][t_capacity][d] contiguous, v_dtype
 *               F32/BF16, 16-byte aligned.
 *   seq_lens    device [n_seq] int32, 0 <= len <= t_capacity.  A sequence of
 *               length 0 yields zeros.
 *   max_len     host: an upper bound of seq_lens (sizes the grid); <= t_capacity.
 *   scale       applied to q . k^ before the softmax (1/sqrt(d) in Alg. 2).
 *   out         device fp32 [n_seq][n_q][n_q_heads][d].
 *   scores_out  device fp32 [n_seq][n_q][n_q_heads][t_capacity] or NULL: the
 *               scaled scores of tokens < len (other entries untouched).
 *   workspace   device, 256-byte aligned, at least
 *               octopus_attn_decode_workspace(...) bytes; contents are scratch.
 * Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP. */
int octopus_attn_decode(const octopus_codebooks_t *cb,
                        const void *q, int32_t q_dtype,
                        int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                        const uint8_t *signs,
                        const void *cache, int64_t t_capacity,
                        const void *v, int32_t v_dtype,
                        const int32_t *seq_lens, int64_t max_len,
                        float scale,
                        float *out, float *scores_out,
                        void *workspace, size_t workspace_bytes,
                        void *stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: octopus_attn_decode without the workspace arguments.  The rotated queries,
 * the split-K partials and the work plan live in a static device array inside the library,
 * OCTOPUS_STATIC_SCRATCH_BYTES bytes on every GPU the library runs on, held until the process ends.  The
 * call allocates and frees nothing (the array's device address is looked up on the first call on a device).
 *   Limit: shapes whose octopus_attn_decode_workspace(...) exceeds OCTOPUS_STATIC_SCRATCH_BYTES are refused
 *   with OCTOPUS_ESCRATCH and nothing is launched (the Llama-shaped decode batch, 16 x 32 heads over 32768
 *   tokens, needs about 19 MiB; a chunk of thousands of query rows does not fit: use octopus_attn_decode).
 *   All calls on one GPU share the one array, which keeps the previous call's contents: calls that overlap
 *   on a GPU (different streams, different threads) race; calls on one stream are ordered and safe.
 * Arguments, results and the other errors are those of octopus_attn_decode, bit for bit. */
#define OCTOPUS_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int octopus_attn_decode_static(const octopus_codebooks_t *cb,
                               const void *q, int32_t q_dtype,
                               int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                               const uint8_t *signs,
                               const void *cache, int64_t t_capacity,
                               const void *v, int32_t v_dtype,
                               const int32_t *seq_lens, int64_t max_len,
                               float scale,
                               float *out, float *scores_out,
                               void *stream);

/* octopus_attn_decode with the QJL-corrected score of Sec. 3.6:
 *   score_t = scale * (q . k^_t + gamma_t * sqrt(pi / (2 d)) * gamma_r,t * (H diag(s') q_rot) . sigma_t),
 * q_rot = H diag(s) q, over a cache and side-car written by octopus_encode_qjl
 * with the same cb, signs and signs2.
 *   signs2, qjl as for octopus_encode_qjl (read only here).
 *   v_dtype     BF16 only (EUNSUPPORTED otherwise).
 * Query rows sharing a KV head (n_q * n_q_heads / n_kv_heads) are served in
 * groups of 8, 4 or 2 rows (the most whose lookup table fits on-chip memory
 * for this head dimension and bit width: 4 at d = 128, b = 3; 2 at d = 256,
 * b = 3); each group reads the head's keys once.  Workspace: octopus_attn_decode_workspace(...) of the
 * same shapes.  Other arguments and errors as octopus_attn_decode; EINVAL if
 * signs2 or qjl is NULL. */
int octopus_attn_decode_qjl(const octopus_codebooks_t *cb,
                            const void *q, int32_t q_dtype,
                            int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                            const uint8_t *signs, const uint8_t *signs2,
                            const void *cache, const void *qjl, int64_t t_capacity,
                            const void *v, int32_t v_dtype,
                            const int32_t *seq_lens, int64_t max_len,
                            float scale,
                            float *out, float *scores_out,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

/* ---- hybrid cache: compressed tokens + a native-precision window (Sec. 4, default recipe) ----
 * The most recent tokens of a sequence are kept uncompressed.  Sequence s holds seq_lens[s]
 * compressed tokens (cache rows 0 .. seq_lens[s]-1) followed by win_lens[s] window tokens whose
 * keys are k_window[s][h][0 .. win_lens[s]-1]; the value buffer holds all of them in order, the
 * window's at rows seq_lens[s] + j.  out = softmax over both parts of scale * q . k (the true key
 * for window tokens, k^ for compressed ones) times the values: the window's partial (m, l, acc)
 * joins the split partials in the merge (flash-decoding identity, App. A).
 *   k_window    device, 16-byte aligned, [n_seq][n_kv_heads][w_capacity][d] contiguous,
 *               k_dtype F32/BF16.
 *   win_lens    device [n_seq] int32, 0 <= win_lens[s] <= w_capacity; window tokens that would
 *               not fit below t_capacity in the value buffer are ignored.
 *   scores_out  window scores are written at positions seq_lens[s] + j.
 * Other arguments, workspace and errors as octopus_attn_decode; EINVAL if k_window or win_lens
 * is NULL or w_capacity < 1.  Moving a token out of the window is an octopus_encode call for it
 * (start_pos = its position) by the caller. */
int octopus_attn_decode_hybrid(const octopus_codebooks_t *cb,
                               const void *q, int32_t q_dtype,
                               int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                               const uint8_t *signs,
                               const void *cache, int64_t t_capacity,
                               const void *v, int32_t v_dtype,
                               const int32_t *seq_lens, int64_t max_len,
                               const void *k_window, int32_t k_dtype, int64_t w_capacity,
                               const int32_t *win_lens,
                               float scale,
                               float *out, float *scores_out,
                               void *workspace, size_t workspace_bytes,
                               void *stream);

/* ---- value codec: per-group quantised values (Sec. 4, "value-side group size in {16, 32}") ----
 * The paper fixes the group size g, the bit width b (that of the keys) and, through the KV
 * ratios of Table (kernel speed), the row size b d / 8 + 8 d / g bytes; the codec is this
 * library's reading: per token, KV head and group of g consecutive channels
 *     lo = min v, hi = max v, scale = (hi - lo) / (2^b - 1) (fp32), zero = lo (fp32),
 *     code_j = clamp(rint((v_j - lo) / scale), 0, 2^b - 1)  (0 when scale = 0; ties to even),
 *     v^_j = zero + scale * code_j.
 * Device layout: [n_seq][n_kv_heads][t_capacity] rows of
 *     [codes: channel j at bit b j of the row, LSB first, b d / 8 bytes][per group: scale, zero]. */

/* Row size in bytes (0 if head_dim is not 64/128/256, bits not 2..4 or group not 16/32). */
size_t octopus_vq_row_bytes(int32_t head_dim, int32_t bits, int32_t group);
/* Bytes of the quantised value buffer (0 if an argument is invalid). */
size_t octopus_vq_bytes(int32_t head_dim, int32_t bits, int32_t group, int32_t n_seq, int32_t n_kv_heads,
                        int64_t t_capacity);

/* Quantises n_new value rows per (sequence, KV head) into rows start_pos[s] + i of vq.
 *   v           device, element (s, i, h, j) at s*stride_seq + i*stride_tok + h*stride_head + j
 *               (element strides), v_dtype F32/BF16, 4-byte aligned.
 *   vq          device, 16-byte aligned, octopus_vq_bytes(...) bytes; other rows untouched.
 *   start_pos   device [n_seq] int32 or NULL (all zero); rows at or past t_capacity are dropped.
 * Errors: EINVAL (also: more than 65535 sequences, or more than 4096 (KV head, group) pairs per token),
 * EUNSUPPORTED (dtype, head_dim, bits, group), EHIP. */
int octopus_encode_values(const void *v, int32_t v_dtype,
                          int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                          int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                          int32_t head_dim, int32_t bits, int32_t group,
                          void *vq, int64_t t_capacity,
                          const int32_t *start_pos,
                          void *stream);

/* octopus_attn_decode over quantised values: out = softmax_t(scale * q . k^_t) V^ with V^ the
 * rows vq dequantised on the fly (the "value dequantization" of Alg. 2).
 *   vq, v_bits, v_group   as written by octopus_encode_values for the same head_dim.
 * Workspace: octopus_attn_decode_workspace(...) of the same shapes.  Other arguments and errors
 * as octopus_attn_decode; EUNSUPPORTED for v_bits outside 2..4 or v_group not 16/32.
 * Without score output (scores_out NULL) the products P.V run on the matrix cores over the codes
 * themselves (output error up to about 1e-4 of a row's largest magnitude); with it, on the vector
 * units over dequantised values (about 1e-5). */
int octopus_attn_decode_vq(const octopus_codebooks_t *cb,
                           const void *q, int32_t q_dtype,
                           int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                           const uint8_t *signs,
                           const void *cache, int64_t t_capacity,
                           const void *vq, int32_t v_bits, int32_t v_group,
                           const int32_t *seq_lens, int64_t max_len,
                           float scale,
                           float *out, float *scores_out,
                           void *workspace, size_t workspace_bytes,
                           void *stream);

/* ---- paged cache (an integration layout; the paper's Sec. 4 recipe leaves the cache's storage open) ----
 * The cache of a sequence need not be contiguous: tokens live in pages of 64 (one tile of the layout
 * above), handed out from pools shared by all sequences, and a block table maps a sequence's logical
 * tile j to its page.  Codes, records and attention are exactly those of octopus_encode /
 * octopus_attn_decode (Alg. 1, Alg. 2); only addresses differ.
 *   k_pool       device, 16-byte aligned: [n_pages][n_kv_heads] key tiles, each the 64-token tile of
 *                the compressed cache layout (granules * 64 * 16 bytes; octopus_paged_pool_bytes).
 *   v_pool       device, 16-byte aligned, bf16: [n_pages][n_kv_heads][64][d] value rows, written by
 *                the caller (token t of a sequence is row t % 64 of page block_table[s][t / 64]).
 *   block_table  device int32 [n_seq][max_pages_per_seq]; entry [s][j] is the page of tokens
 *                64 j .. 64 j + 63 of sequence s.  Only entries below ceil(len / 64) are read.  Ids
 *                are clamped to [0, n_pages): a wrong table yields wrong results, never an access
 *                outside the pools.  Two sequences may share a page (a common prefix).
 * octopus_encode_paged: arguments as octopus_encode with (cache, t_capacity) replaced by the pool and
 * the table; a sequence can hold max_pages_per_seq * 64 tokens, tokens past that are dropped.
 * octopus_attn_decode_paged: arguments as octopus_attn_decode (bf16 values only, no scores_out);
 * max_len <= max_pages_per_seq * 64; query rows are served in groups of at most 8 per KV head, 32 or more
 * query rows per KV head (n_q * n_q_heads / n_kv_heads) by the many-row kernel up to head_dim 128 and refused
 * with EUNSUPPORTED at head_dim 256 (as hundreds of row groups each would read the keys again).
 * Workspace: octopus_attn_decode_workspace of the same shapes.  Errors: EINVAL for NULL / misaligned pointers, n_pages < 1, max_pages_per_seq < 1 and the
 * conditions of the contiguous calls; EUNSUPPORTED / EWORKSPACE / EHIP as there. */
size_t octopus_paged_pool_bytes(const octopus_codebooks_t *cb, int32_t n_pages, int32_t n_kv_heads);

int octopus_encode_paged(const octopus_codebooks_t *cb,
                         const void *keys, int32_t key_dtype,
                         int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                         int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                         const uint8_t *signs,
                         void *k_pool, int32_t n_pages,
                         const int32_t *block_table, int32_t max_pages_per_seq,
                         const int32_t *start_pos,
                         void *stream);

int octopus_attn_decode_paged(const octopus_codebooks_t *cb,
                              const void *q, int32_t q_dtype,
                              int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                              const uint8_t *signs,
                              const void *k_pool, const void *v_pool, int32_t n_pages,
                              const int32_t *block_table, int32_t max_pages_per_seq,
                              const int32_t *seq_lens, int64_t max_len,
                              float scale,
                              float *out,
                              void *workspace, size_t workspace_bytes,
                              void *stream);

/* octopus_attn_decode_paged plus the native-precision window of octopus_attn_decode_hybrid (Sec. 4,
 * default recipe): sequence s holds seq_lens[s] compressed tokens in its key pages, followed by
 * win_lens[s] window tokens whose keys are k_window[s][h][0 .. win_lens[s]-1]; the value rows of ALL
 * its tokens lie in its value pages, the window's at positions seq_lens[s] + j (row (seq_lens[s] + j) % 64
 * of page block_table[s][(seq_lens[s] + j) / 64]).  Window tokens at or past max_pages_per_seq * 64 are
 * ignored.  k_window, k_dtype, w_capacity, win_lens as for octopus_attn_decode_hybrid; everything else,
 * the limits and the errors as for octopus_attn_decode_paged; EINVAL if k_window or win_lens is NULL
 * or w_capacity < 1. */
int octopus_attn_decode_paged_hybrid(const octopus_codebooks_t *cb,
                                     const void *q, int32_t q_dtype,
                                     int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                                     const uint8_t *signs,
                                     const void *k_pool, const void *v_pool, int32_t n_pages,
                                     const int32_t *block_table, int32_t max_pages_per_seq,
                                     const int32_t *seq_lens, int64_t max_len,
                                     const void *k_window, int32_t k_dtype, int64_t w_capacity,
                                     const int32_t *win_lens,
                                     float scale,
                                     float *out,
                                     void *workspace, size_t workspace_bytes,
                                     void *stream);

/* Group-quantised values (octopus_encode_values, octopus_attn_decode_vq) in pages.
 *   vq_pool     device, 16-byte aligned: [n_pages][n_kv_heads][64] rows of octopus_vq_row_bytes(head_dim,
 *               bits, group) bytes (octopus_vq_bytes(head_dim, bits, group, n_pages, n_kv_heads, 64) in all);
 *               token t of sequence s is row t % 64 of page block_table[s][t / 64].
 * octopus_encode_values_paged: arguments as octopus_encode_values with (vq, t_capacity) replaced by the pool
 * and the table; rows at or past max_pages_per_seq * 64 are dropped; the rows written are byte for byte those
 * of octopus_encode_values.
 * octopus_attn_decode_paged_vq: octopus_attn_decode_paged over such a pool instead of bf16 value pages
 * (v_bits, v_group as for octopus_attn_decode_vq).  Served by the matrix-core kernel only: shapes it is not
 * built for (octopus_vq_on_matrix_cores(...) == 0) are refused with EUNSUPPORTED, as are 32 or more query
 * rows per KV head (with quantised values or the QJL side-car over pages).  Other arguments, workspace and
 * errors as octopus_attn_decode_paged. */
int octopus_encode_values_paged(const void *v, int32_t v_dtype,
                                int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                                int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                                int32_t head_dim, int32_t bits, int32_t group,
                                void *vq_pool, int32_t n_pages,
                                const int32_t *block_table, int32_t max_pages_per_seq,
                                const int32_t *start_pos,
                                void *stream);

int octopus_attn_decode_paged_vq(const octopus_codebooks_t *cb,
                                 const void *q, int32_t q_dtype,
                                 int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                                 const uint8_t *signs,
                                 const void *k_pool, const void *vq_pool, int32_t v_bits, int32_t v_group,
                                 int32_t n_pages,
                                 const int32_t *block_table, int32_t max_pages_per_seq,
                                 const int32_t *seq_lens, int64_t max_len,
                                 float scale,
                                 float *out,
                                 void *workspace, size_t workspace_bytes,
                                 void *stream);

/* The 1-bit QJL residual (octopus_encode_qjl, octopus_attn_decode_qjl) in pages.
 *   qjl_pool    device, 4-byte aligned: [n_pages][n_kv_heads] side-car tiles of 64 tokens, each laid out
 *               as a tile of the contiguous side-car (octopus_qjl_bytes(cb, n_pages, n_kv_heads, 64) in all);
 *               the tile of tokens 64 j .. 64 j + 63 of sequence s is that of page block_table[s][j].
 * octopus_encode_qjl_paged: octopus_encode_paged that also writes the side-car (signs2 as for
 * octopus_encode_qjl); codes and side-car are byte for byte those of octopus_encode_qjl.
 * octopus_attn_decode_paged_qjl: octopus_attn_decode_paged with the corrected score of
 * octopus_attn_decode_qjl (bf16 value pages; row groups as there; 32 or more query rows per KV head are
 * refused with EUNSUPPORTED).  EINVAL if signs2 or qjl_pool is NULL;
 * other arguments, workspace and errors as octopus_encode_paged / octopus_attn_decode_paged. */
int octopus_encode_qjl_paged(const octopus_codebooks_t *cb,
                             const void *keys, int32_t key_dtype,
                             int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                             int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                             const uint8_t *signs, const uint8_t *signs2,
                             void *k_pool, void *qjl_pool, int32_t n_pages,
                             const int32_t *block_table, int32_t max_pages_per_seq,
                             const int32_t *start_pos,
                             void *stream);

int octopus_attn_decode_paged_qjl(const octopus_codebooks_t *cb,
                                  const void *q, int32_t q_dtype,
                                  int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                                  const uint8_t *signs, const uint8_t *signs2,
                                  const void *k_pool, const void *qjl_pool, const void *v_pool, int32_t n_pages,
                                  const int32_t *block_table, int32_t max_pages_per_seq,
                                  const int32_t *seq_lens, int64_t max_len,
                                  float scale,
                                  float *out,
                                  void *workspace, size_t workspace_bytes,
                                  void *stream);

/* Static, human-readable name of an error code. */
const char *octopus_strerror(int code);

/* ---- measurement aids (not part of the method; nothing above depends on them) ----
 * octopus_profile_events: the next decode-attention call made by this thread (octopus_attn_decode, its _static,
 * _qjl, _vq and _hybrid forms, octopus_attn_decode_paged and its _hybrid, _vq and _qjl forms) records the HIP events `before` and `after` (hipEvent_t
 * passed as void*, caller-owned, created with timing enabled) on the call's stream immediately before and after
 * the launch of its fused decode kernel, i.e. around Alg. 2 proper without the query rotation and the split
 * merge.  The handles are per thread and are forgotten by that call whether it succeeds or not; NULL, NULL
 * cancels.  Returns OCTOPUS_OK, or OCTOPUS_EINVAL if only one of the two is NULL. */
int octopus_profile_events(void *before, void *after);

/* octopus_vq_on_matrix_cores: 1 if octopus_attn_decode_vq without score output serves this shape and value
 * format with the kernel that multiplies P.V on the matrix cores, 0 if with the vector-unit kernel (or if the
 * arguments are not ones the call accepts).  Host-side; says which kernel a measurement is of. */
int octopus_vq_on_matrix_cores(const octopus_codebooks_t *cb, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                               int32_t v_bits, int32_t v_group);

/* octopus_probe_read: a plain streaming read of `bytes` bytes of device memory at `data` (16-byte aligned) by
 * n_workgroups workgroups of 256 threads, each walking its contiguous share with 16-byte loads, non-temporal or
 * not: the reference that says what read rate the machine reaches with nothing else to do.  `sink`: 4 bytes of
 * device memory (practically never written).  Errors: EINVAL, EHIP. */
int octopus_probe_read(const void *data, size_t bytes, int32_t nontemporal, int32_t n_workgroups, void *sink,
                       void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OCTOPUS_H_ */
