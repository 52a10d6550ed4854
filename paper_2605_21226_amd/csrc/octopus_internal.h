// Internal declarations shared by the host dispatch code and the HIP kernels.
#ifndef OCTOPUS_INTERNAL_H_
#define OCTOPUS_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include "octopus.h"

namespace octopus {

// Centroids handed to kernels by value (kernel argument space); boundaries are
// recomputed on the device as midpoints, exactly as the host computes them.
constexpr int kMaxLevels = OCTOPUS_MAX_LEVELS;   // 64: up to 6 bits per index (the pairs swept in App. D)
struct DeviceBooks {
    float c_xi[2][kMaxLevels];
    float c_rho[2][kMaxLevels];
};

inline DeviceBooks device_books(const octopus_codebooks_t &cb) {
    DeviceBooks books;
    for (int c = 0; c < 2; ++c)
        for (int k = 0; k < kMaxLevels; ++k) {
            books.c_xi[c][k] = cb.c_xi[c][k];
            books.c_rho[c][k] = cb.c_rho[c][k];
        }
    return books;
}

// Floats per rotated query row in the workspace: 3 * n_tri rounded up to 4.
inline int q_row_stride(int n_tri) { return (3 * n_tri + 3) & ~3; }

struct DecodeShape {
    int32_t n_seq, n_q_heads, n_kv_heads, n_q;
    int32_t heads_per_kv;   // n_q_heads / n_kv_heads
    int32_t rows_per_kv;    // n_q * heads_per_kv query rows sharing one KV head
    int32_t rows_per_pass;  // query rows one workgroup scores per key (1, 2, 4 or 8; 128 or 256: many-row kernel)
    int32_t n_row_groups;   // ceil(rows_per_kv / rows_per_pass)
    int32_t n_splits;       // wavefronts (workgroups of the many-row kernel) sharing the tiles of one (sequence, KV head, row group)
    int32_t max_items;      // bound of the work items the device cuts (row groups of at most 8)
    int32_t max_len;        // host-side bound of the sequence lengths
    int32_t item_waves;     // wavefronts of the workgroup that share a work item (4; 8: matrix-core kernel over quantised values up to d = 128 where its LDS fits)
    int32_t tiles_per_step; // 64-token tiles a wavefront takes per step (2 up to d = 128, else 1; 1: that kernel)
    int64_t t_capacity;
};

// Paged cache: logical 64-token tile j of sequence s lives in page table[s * stride + j] of a pool of n_pages
// pages; table NULL: the contiguous cache.
struct PageTable {
    const int32_t *table;
    int32_t stride;
    int32_t n_pages;
};

// Workspace carve-up (all offsets multiples of 256 bytes).
struct Workspace {
    size_t q_rot_off, part_ml_off, part_acc_off, plan_off, q2_off, win_ml_off, win_acc_off, total;
};

DecodeShape make_decode_shape(const octopus_plan_t &plan, int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t n_q, int64_t max_len, int64_t t_capacity, bool many_rows, int32_t rows_cap = 8,
                              int32_t vq_mfma_waves = 0);
// Row group the matrix-core kernel over quantised values would serve a call with (4 or 8 query rows), and
// whether such a kernel is built for the plan and value format (octopus_common.hip).
inline int32_t vq_mfma_rows(int32_t rows_per_kv) { return rows_per_kv <= 4 ? 4 : 8; }
// wavefronts per workgroup (4 or 8) of the matrix-core kernel over quantised values built for the shape, 0: none
int vq_mfma_available(const octopus_plan_t &plan, int32_t rows_per_pass, int32_t v_bits, int32_t v_group);
Workspace make_workspace(const octopus_plan_t &plan, const DecodeShape &s);

// Kernel launchers (defined in the .hip files).  Each returns a hipError_t cast to int.
// `work_plan`: device array the rotation kernel fills with the work items of the split-K kernel (NULL with
// the many-row kernel, whose blocks are split on the host).  `q2` (NULL: not wanted): the queries rotated a second time
// with `signs2` for the QJL residual, [padded row][head_dim].
int launch_rotate_queries(const octopus_plan_t &plan, const void *q, int q_dtype, const uint8_t *signs,
                          const DecodeShape &s, float scale, float *q_rot, const int32_t *seq_lens,
                          int32_t *work_plan, const uint8_t *signs2, float *q2, void *stream);
int launch_decode(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                  const void *v, int v_dtype, const int32_t *seq_lens, float *part_ml, float *part_acc,
                  float *scores_out, int32_t *work_plan, void *stream);
// bf16 values, row groups of at most qjl_rows_cap(plan)
int launch_decode_qjl(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                      const void *qjl, const float *q2, const void *v, const int32_t *seq_lens, float *part_ml,
                      float *part_acc, float *scores_out, int32_t *work_plan, void *stream);
// Query rows one workgroup of the QJL decode kernel serves: the largest of 8, 4, 2, 1 whose sign-byte table
// fits LDS beside the plan's decode tables; 0 if the plan is not built.
int qjl_rows_cap(const octopus_plan_t &plan);
// win_ml / win_acc: the partial of a native-precision window per output row, or NULL
int launch_merge(const octopus_plan_t &plan, const DecodeShape &s, const float *part_ml, const float *part_acc,
                 const int32_t *work_plan, float *out, const float *win_ml, const float *win_acc, void *stream);
// Attention partial (m, l, acc) per output row over the native-precision window that follows the
// compressed tokens of each sequence; pt: the value rows lie in pages (s.t_capacity = what the table addresses).
int launch_window(const octopus_plan_t &plan, const DecodeShape &s, const void *q, int q_dtype, const void *k_win,
                  int k_dtype, int64_t w_capacity, const int32_t *win_lens, const void *v, int v_dtype,
                  const int32_t *seq_lens, float scale, float *win_ml, float *win_acc, float *scores_out,
                  void *stream, PageTable pt = PageTable{nullptr, 0, 0});
int launch_encode(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                  int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                  const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                  const uint8_t *signs2, void *qjl, void *stream);   // qjl NULL: no side-car

// Paged pools: the encoder writes each tile into its page of `k_pool` ([page][KV head] key tiles); the decode
// kernel reads key tiles from `k_pool` and bf16 value tiles ([page][KV head][64][head_dim]) from `v_pool`.
int launch_encode_paged(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                        int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                        const uint8_t *signs, void *k_pool, const PageTable &pt, const int32_t *start_pos,
                        void *stream, const uint8_t *signs2 = nullptr, void *qjl_pool = nullptr);   // qjl_pool: side-car pages
int launch_decode_paged(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *k_pool,
                        const void *v_pool, const PageTable &pt, const int32_t *seq_lens, float *part_ml,
                        float *part_acc, int32_t *work_plan, void *stream);
// ... with the QJL side-car in pages as well ([page][KV head] side-car tiles), q2 as for launch_decode_qjl
int launch_decode_paged_qjl(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *k_pool,
                            const void *qjl_pool, const float *q2, const void *v_pool, const PageTable &pt,
                            const int32_t *seq_lens, float *part_ml, float *part_acc, int32_t *work_plan, void *stream);

// The encoder with one of the rounding modes of App. E (OCTOPUS_ROUND_*), no side-car.
int launch_encode_rounding(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                           int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                           const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                           int32_t mode, void *stream);

// Value codec (group-quantised value rows) and decode attention over it.
int launch_encode_values(const void *v, int v_dtype, int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                         int32_t n_seq, int32_t n_kv_heads, int32_t n_new, int32_t head_dim, int32_t bits,
                         int32_t group, void *vq, int64_t t_capacity, const int32_t *start_pos, void *stream,
                         PageTable pt = PageTable{nullptr, 0, 0});   // pt: vq is a pool of [page][KV head][64] rows
int launch_decode_vq(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                     const void *vq, int v_bits, int v_group, const int32_t *seq_lens, float *part_ml,
                     float *part_acc, float *scores_out, int32_t *work_plan, void *stream,
                     PageTable pt = PageTable{nullptr, 0, 0});   // pt: cache and vq are pools of pages

// Measurement aid: plain streaming read of `bytes` bytes by n_blocks workgroups (non-temporal loads or not).
int launch_probe_read(const void *data, int64_t bytes, int nontemporal, int n_blocks, void *sink, void *stream);

// hipEventRecord(event, stream); returns a hipError_t cast to int.
int record_event(void *event, void *stream);

// True when every kernel family is instantiated for this plan (the six built bit widths of each head dimension).
bool plan_supported(const octopus_plan_t &plan);
// True for the extra (b_dir, b_nrm) pairs of the App. D sweep: plain encoder (local 3x3) and split-K decode over
// bf16 values only -- no score output, no QJL side-car, no quantised values, no pages, no many-row kernel.
bool plan_sweep_only(const octopus_plan_t &plan);

}  // namespace octopus

#endif
