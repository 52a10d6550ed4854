// Dispatch by head dimension and the kernels that do not depend on the bit width.
#include "octopus_decode.hpp"
#include "octopus_window.hpp"

namespace octopus {

bool plan_supported_d64(const octopus_plan_t &);
bool plan_supported_d128(const octopus_plan_t &);
bool plan_supported_d256(const octopus_plan_t &);
#define OCTOPUS_DECL(D)                                                                                            \
    int launch_decode_mfma_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *,     \
                                const void *, const int32_t *, float *, float *, float *, int32_t *, void *);      \
    int launch_decode_mfma_scores_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *,            \
                                       const void *, const void *, const int32_t *, float *, float *, float *,     \
                                       int32_t *, void *);                                                         \
    int launch_decode_valu_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *,     \
                                const void *, const int32_t *, float *, float *, float *, int32_t *, void *);      \
    int launch_encode_d##D(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t, int32_t,     \
                           int32_t, int32_t, const uint8_t *, void *, int64_t, const int32_t *, const uint8_t *, void *, \
                           void *);                                                                                \
    int launch_decode_qjl_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *,      \
                               const void *, const float *, const void *, const int32_t *, float *, float *,       \
                               float *, int32_t *, void *);                                                        \
    int qjl_rows_cap_d##D(const octopus_plan_t &);                                                                 \
    int vq_mfma_available_d##D(const octopus_plan_t &, int, int, int);                                             \
    int launch_decode_vq_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *,       \
                              const void *, int, int, const int32_t *, float *, float *, float *, int32_t *,       \
                              void *, const PageTable &);                                                          \
    int launch_encode_rounding_d##D(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t,     \
                                    int32_t, int32_t, int32_t, const uint8_t *, void *, int64_t, const int32_t *,  \
                                    int32_t, void *);                                                              \
    int launch_decode_paged_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *,    \
                                 const void *, const PageTable &, const int32_t *, float *, float *, int32_t *,    \
                                 void *);                                                                          \
    int launch_encode_paged_d##D(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t,        \
                                 int32_t, int32_t, int32_t, const uint8_t *, void *, const PageTable &,            \
                                 const int32_t *, const uint8_t *, void *, void *);                                \
    int launch_decode_paged_qjl_d##D(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, \
                                     const void *, const float *, const void *, const PageTable &, const int32_t *, \
                                     float *, float *, int32_t *, void *);
OCTOPUS_DECL(64)
OCTOPUS_DECL(128)
OCTOPUS_DECL(256)
#undef OCTOPUS_DECL

// Measurement aid: a plain streaming read of `bytes` bytes (16 bytes per lane, every workgroup walks its own
// contiguous share front to back, 8 loads in flight per lane), with or without the non-temporal hint.
template <bool NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint32_t *__restrict__ p, int64_t units_per_block,
                                                         uint32_t *__restrict__ sink) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t *base = reinterpret_cast<const u32x4_t *>(p) + static_cast<int64_t>(blockIdx.x) * units_per_block;
    uint32_t acc = 0;
    for (int64_t i = threadIdx.x; i < units_per_block; i += 256 * 8) {
        u32x4_t x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t j = min(i + u * 256, units_per_block - 1);
            x[u] = NT ? __builtin_nontemporal_load(base + j) : base[j];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;   // (keeps the loads alive; practically never taken)
}

int launch_probe_read(const void *data, int64_t bytes, int nontemporal, int n_blocks, void *sink, void *stream) {
    const int64_t units = bytes / 16 / n_blocks;
    if (nontemporal)
        hipLaunchKernelGGL(probe_read_kernel<true>, dim3(n_blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                           static_cast<const uint32_t *>(data), units, static_cast<uint32_t *>(sink));
    else
        hipLaunchKernelGGL(probe_read_kernel<false>, dim3(n_blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                           static_cast<const uint32_t *>(data), units, static_cast<uint32_t *>(sink));
    return static_cast<int>(hipGetLastError());
}

// the pairs of the App. D sweep (head dimension 128 only): plain encoder and bf16-value split-K decode
bool plan_supported_sweep_d128(const octopus_plan_t &);
int launch_decode_sweep_d128(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *,
                             const int32_t *, float *, float *, int32_t *, void *);
int launch_encode_sweep_d128(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t, int32_t, int32_t,
                             int32_t, const uint8_t *, void *, int64_t, const int32_t *, void *);

int record_event(void *event, void *stream) {
    return static_cast<int>(hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)));
}

bool plan_sweep_only(const octopus_plan_t &plan) { return plan.head_dim == 128 && plan_supported_sweep_d128(plan); }

bool plan_supported(const octopus_plan_t &plan) {
    switch (plan.head_dim) {
        case 64: return plan_supported_d64(plan);
        case 128: return plan_supported_d128(plan);
        case 256: return plan_supported_d256(plan);
        default: return false;
    }
}

int launch_decode(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                  const void *v, int v_dtype, const int32_t *seq_lens, float *part_ml, float *part_acc,
                  float *scores_out, int32_t *work_plan, void *stream) {
    if (plan_sweep_only(cb.plan)) {
        if (v_dtype != OCTOPUS_DTYPE_BF16 || scores_out != nullptr) return static_cast<int>(hipErrorInvalidValue);
        return launch_decode_sweep_d128(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, work_plan, stream);
    }
    // kernel family: 0 matrix cores, 1 matrix cores with score output, 2 vector units (fp32 values)
    const int family = v_dtype == OCTOPUS_DTYPE_BF16 ? (scores_out != nullptr ? 1 : 0) : 2;
#define OCTOPUS_GO(D)                                                                                                   \
    case D:                                                                                                             \
        return family == 0   ? launch_decode_mfma_d##D(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out,  \
                                                       work_plan, stream)                                               \
               : family == 1 ? launch_decode_mfma_scores_d##D(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc,       \
                                                              scores_out, work_plan, stream)                            \
                             : launch_decode_valu_d##D(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out,  \
                                                       work_plan, stream);
    switch (cb.plan.head_dim) {
        OCTOPUS_GO(64)
        OCTOPUS_GO(128)
        OCTOPUS_GO(256)
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef OCTOPUS_GO
}

int launch_decode_vq(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                     const void *vq, int v_bits, int v_group, const int32_t *seq_lens, float *part_ml,
                     float *part_acc, float *scores_out, int32_t *work_plan, void *stream, PageTable pt) {
    switch (cb.plan.head_dim) {
        case 64: return launch_decode_vq_d64(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, work_plan, stream, pt);
        case 128: return launch_decode_vq_d128(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, work_plan, stream, pt);
        case 256: return launch_decode_vq_d256(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, work_plan, stream, pt);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int vq_mfma_available(const octopus_plan_t &plan, int32_t rows_per_pass, int32_t v_bits, int32_t v_group) {
    if (plan_sweep_only(plan)) return 0;
    switch (plan.head_dim) {
        case 64: return vq_mfma_available_d64(plan, rows_per_pass, v_bits, v_group);
        case 128: return vq_mfma_available_d128(plan, rows_per_pass, v_bits, v_group);
        case 256: return vq_mfma_available_d256(plan, rows_per_pass, v_bits, v_group);
        default: return 0;
    }
}

int qjl_rows_cap(const octopus_plan_t &plan) {
    switch (plan.head_dim) {
        case 64: return qjl_rows_cap_d64(plan);
        case 128: return qjl_rows_cap_d128(plan);
        case 256: return qjl_rows_cap_d256(plan);
        default: return 0;
    }
}

int launch_decode_qjl(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                      const void *qjl, const float *q2, const void *v, const int32_t *seq_lens, float *part_ml,
                      float *part_acc, float *scores_out, int32_t *work_plan, void *stream) {
    switch (cb.plan.head_dim) {
        case 64: return launch_decode_qjl_d64(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, work_plan, stream);
        case 128: return launch_decode_qjl_d128(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, work_plan, stream);
        case 256: return launch_decode_qjl_d256(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, work_plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int launch_encode(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                  int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                  const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                  const uint8_t *signs2, void *qjl, void *stream) {
    if (plan_sweep_only(cb.plan)) {
        if (qjl != nullptr) return static_cast<int>(hipErrorInvalidValue);
        return launch_encode_sweep_d128(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new,
                                        signs, cache, t_capacity, start_pos, stream);
    }
    switch (cb.plan.head_dim) {
        case 64: return launch_encode_d64(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, signs2, qjl, stream);
        case 128: return launch_encode_d128(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, signs2, qjl, stream);
        case 256: return launch_encode_d256(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, signs2, qjl, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int launch_decode_paged(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *k_pool,
                        const void *v_pool, const PageTable &pt, const int32_t *seq_lens, float *part_ml,
                        float *part_acc, int32_t *work_plan, void *stream) {
    switch (cb.plan.head_dim) {
        case 64: return launch_decode_paged_d64(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        case 128: return launch_decode_paged_d128(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        case 256: return launch_decode_paged_d256(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int launch_encode_paged(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                        int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                        const uint8_t *signs, void *k_pool, const PageTable &pt, const int32_t *start_pos,
                        void *stream, const uint8_t *signs2, void *qjl_pool) {
    switch (cb.plan.head_dim) {
        case 64: return launch_encode_paged_d64(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, k_pool, pt, start_pos, signs2, qjl_pool, stream);
        case 128: return launch_encode_paged_d128(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, k_pool, pt, start_pos, signs2, qjl_pool, stream);
        case 256: return launch_encode_paged_d256(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, k_pool, pt, start_pos, signs2, qjl_pool, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int launch_decode_paged_qjl(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *k_pool,
                            const void *qjl_pool, const float *q2, const void *v_pool, const PageTable &pt,
                            const int32_t *seq_lens, float *part_ml, float *part_acc, int32_t *work_plan, void *stream) {
    switch (cb.plan.head_dim) {
        case 64: return launch_decode_paged_qjl_d64(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        case 128: return launch_decode_paged_qjl_d128(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        case 256: return launch_decode_paged_qjl_d256(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

int launch_encode_rounding(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                           int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                           const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                           int32_t mode, void *stream) {
    switch (cb.plan.head_dim) {
        case 64: return launch_encode_rounding_d64(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, mode, stream);
        case 128: return launch_encode_rounding_d128(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, mode, stream);
        case 256: return launch_encode_rounding_d256(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, cache, t_capacity, start_pos, mode, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

template <int D>
static int rotate_d(const void *q, int q_dtype, const uint8_t *signs, const DecodeShape &s, float scale, float *q_rot,
                    const int32_t *seq_lens, int32_t *work_plan, const uint8_t *signs2, float *q2,
                    hipStream_t stream) {
    constexpr int QS = (3 * ((D + 2) / 3) + 3) & ~3;
    const int64_t rows = static_cast<int64_t>(s.n_seq) * s.n_kv_heads * s.n_row_groups * s.rows_per_pass;
    hipLaunchKernelGGL((rotate_queries_kernel<D, QS>), dim3(static_cast<unsigned>(rows)), dim3(kWave), 0, stream, q,
                       q_dtype == OCTOPUS_DTYPE_BF16 ? 1 : 0, signs, s, scale, q_rot, seq_lens, work_plan, signs2, q2);
    return static_cast<int>(hipGetLastError());
}

int launch_rotate_queries(const octopus_plan_t &plan, const void *q, int q_dtype, const uint8_t *signs,
                          const DecodeShape &s, float scale, float *q_rot, const int32_t *seq_lens,
                          int32_t *work_plan, const uint8_t *signs2, float *q2, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (plan.head_dim) {
        case 64: return rotate_d<64>(q, q_dtype, signs, s, scale, q_rot, seq_lens, work_plan, signs2, q2, st);
        case 128: return rotate_d<128>(q, q_dtype, signs, s, scale, q_rot, seq_lens, work_plan, signs2, q2, st);
        case 256: return rotate_d<256>(q, q_dtype, signs, s, scale, q_rot, seq_lens, work_plan, signs2, q2, st);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

template <int D>
static int merge_d(const DecodeShape &s, const float *part_ml, const float *part_acc, const int32_t *work_plan,
                   float *out, const float *win_ml, const float *win_acc, hipStream_t stream) {
    const int64_t rows = static_cast<int64_t>(s.n_seq) * s.n_q * s.n_q_heads;
    hipLaunchKernelGGL((merge_kernel<D>), dim3(static_cast<unsigned>(rows)), dim3(kWave), 0, stream, s, part_ml,
                       part_acc, work_plan, out, win_ml, win_acc);
    return static_cast<int>(hipGetLastError());
}

int launch_merge(const octopus_plan_t &plan, const DecodeShape &s, const float *part_ml, const float *part_acc,
                 const int32_t *work_plan, float *out, const float *win_ml, const float *win_acc, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (plan.head_dim) {
        case 64: return merge_d<64>(s, part_ml, part_acc, work_plan, out, win_ml, win_acc, st);
        case 128: return merge_d<128>(s, part_ml, part_acc, work_plan, out, win_ml, win_acc, st);
        case 256: return merge_d<256>(s, part_ml, part_acc, work_plan, out, win_ml, win_acc, st);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

template <int D>
static int window_d(const DecodeShape &s, const void *q, int q_dtype, const void *k_win, int k_dtype,
                    int64_t w_capacity, const int32_t *win_lens, const void *v, int v_dtype, const int32_t *seq_lens,
                    float scale, float *win_ml, float *win_acc, float *scores_out, PageTable pt, hipStream_t stream) {
    const int64_t rows = static_cast<int64_t>(s.n_seq) * s.n_q * s.n_q_heads;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(rows)), dim3(kWave), 0, stream, s, q,
                           q_dtype == OCTOPUS_DTYPE_BF16 ? 1 : 0, k_win, w_capacity, win_lens, v, seq_lens, scale, win_ml,
                           win_acc, scores_out, pt);
    };
    const bool kb = k_dtype == OCTOPUS_DTYPE_BF16, vb = v_dtype == OCTOPUS_DTYPE_BF16;
    if (kb && vb) go(window_kernel<D, true, true>);
    else if (kb) go(window_kernel<D, true, false>);
    else if (vb) go(window_kernel<D, false, true>);
    else go(window_kernel<D, false, false>);
    return static_cast<int>(hipGetLastError());
}

int launch_window(const octopus_plan_t &plan, const DecodeShape &s, const void *q, int q_dtype, const void *k_win,
                  int k_dtype, int64_t w_capacity, const int32_t *win_lens, const void *v, int v_dtype,
                  const int32_t *seq_lens, float scale, float *win_ml, float *win_acc, float *scores_out,
                  void *stream, PageTable pt) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (plan.head_dim) {
        case 64: return window_d<64>(s, q, q_dtype, k_win, k_dtype, w_capacity, win_lens, v, v_dtype, seq_lens, scale, win_ml, win_acc, scores_out, pt, st);
        case 128: return window_d<128>(s, q, q_dtype, k_win, k_dtype, w_capacity, win_lens, v, v_dtype, seq_lens, scale, win_ml, win_acc, scores_out, pt, st);
        case 256: return window_d<256>(s, q, q_dtype, k_win, k_dtype, w_capacity, win_lens, v, v_dtype, seq_lens, scale, win_ml, win_acc, scores_out, pt, st);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace octopus
