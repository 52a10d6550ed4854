// Native-precision window of a hybrid cache (Sec. 4, default recipe: a short residual window of recent
// tokens kept uncompressed).  The window's tokens follow the compressed ones of their sequence; their
// keys are read as stored, their scores are the plain scale * q . k, and the partial (m, l, acc) of the
// window joins the split partials of the compressed part in the merge (flash-decoding identity, App. A).
#ifndef OCTOPUS_WINDOW_HPP_
#define OCTOPUS_WINDOW_HPP_

#include "octopus_decode.hpp"

namespace octopus {

// One wavefront per output row (sequence, query, query head).  Keys: [n_seq][n_kv_heads][w_capacity][D],
// values: rows seq_lens[s] + j of the value buffer [n_seq][n_kv_heads][t_capacity][D] (bf16 or fp32 each); with a
// page table (pt.table not NULL) token t of sequence s is row t % 64 of [page][KV head] of a pool of value pages,
// page = pt.table[s * pt.stride + t / 64] clamped to the pool, and t_capacity is what the table can address.
// Chunks of 64 window tokens, one token per lane for the scores (the query sits in LDS), then every lane
// accumulates its D / 64 channels over the chunk's tokens.
template <int D, bool k_is_bf16, bool v_is_bf16>
__global__ __launch_bounds__(kWave) void window_kernel(DecodeShape shp, const void *__restrict__ q, int q_is_bf16,
                                                       const void *__restrict__ k_win,
                                                       int64_t w_capacity, const int32_t *__restrict__ win_lens,
                                                       const void *__restrict__ v,
                                                       const int32_t *__restrict__ seq_lens, float scale,
                                                       float *__restrict__ win_ml, float *__restrict__ win_acc,
                                                       float *__restrict__ scores_out, PageTable pt) {
    constexpr int CPT = D / kWave;  // channels per lane: c * 64 + lane
    __shared__ float qs[D];
    const int lane = threadIdx.x;
    const int64_t orow = blockIdx.x;  // (seq, qi, head)
    const int head = static_cast<int>(orow % shp.n_q_heads);
    const int seq = static_cast<int>(orow / (static_cast<int64_t>(shp.n_q_heads) * shp.n_q));
    const int kvh = head / shp.heads_per_kv;
    auto load = [](const void *p, int is_bf16, int64_t i) {
        return is_bf16 ? __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(p)[i]) << 16)
                       : static_cast<const float *>(p)[i];
    };
#pragma unroll
    for (int c = 0; c < CPT; ++c) qs[c * kWave + lane] = load(q, q_is_bf16, orow * D + c * kWave + lane) * scale;
    __syncthreads();

    const int64_t len = min(max(seq_lens[seq], 0), shp.max_len);   // clamped like every other kernel's
    // the window's tokens must fit behind the compressed ones in the value buffer
    const int64_t n_win = max(int64_t{0}, min(min(static_cast<int64_t>(win_lens[seq]), w_capacity), shp.t_capacity - len));
    const int64_t pair = static_cast<int64_t>(seq) * shp.n_kv_heads + kvh;
    const int64_t k_row0 = pair * w_capacity, v_row0 = pair * shp.t_capacity + len;
    // row of the value buffer (or pool) that holds window token j
    auto v_row = [&](int64_t j) -> int64_t {
        if (pt.table == nullptr) return v_row0 + j;
        const int64_t t = len + j;
        const int page = pt.table[static_cast<int64_t>(seq) * pt.stride + t / kWave];
        return (static_cast<int64_t>(min(max(page, 0), pt.n_pages - 1)) * shp.n_kv_heads + kvh) * kWave + t % kWave;
    };

    float m_run = -INFINITY, l_run = 0.0f, acc[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) acc[c] = 0.0f;
    for (int64_t j0 = 0; j0 < n_win; j0 += kWave) {
        const int nj = static_cast<int>(min(static_cast<int64_t>(kWave), n_win - j0));
        float s = -INFINITY;
        if (lane < nj) {
            // this lane's key row, 16 bytes at a time (rows are 2 D or 4 D bytes: multiples of 16)
            float dot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            const int64_t kb = (k_row0 + j0 + lane) * D;
            if (k_is_bf16) {
                const uint4 *kp = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(k_win) + kb);
#pragma unroll
                for (int e = 0; e < D / 8; ++e) {
                    const uint4 x = kp[e];
                    const uint32_t w4[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        dot[h] = fmaf(qs[8 * e + 2 * h], __uint_as_float(w4[h] << 16), dot[h]);
                        dot[h] = fmaf(qs[8 * e + 2 * h + 1], __uint_as_float(w4[h] & 0xffff0000u), dot[h]);
                    }
                }
            } else {
                const float4 *kp = reinterpret_cast<const float4 *>(static_cast<const float *>(k_win) + kb);
#pragma unroll 16
                for (int e = 0; e < D / 4; ++e) {
                    const float4 x = kp[e];
                    dot[0] = fmaf(qs[4 * e], x.x, dot[0]);
                    dot[1] = fmaf(qs[4 * e + 1], x.y, dot[1]);
                    dot[2] = fmaf(qs[4 * e + 2], x.z, dot[2]);
                    dot[3] = fmaf(qs[4 * e + 3], x.w, dot[3]);
                }
            }
            s = (dot[0] + dot[1]) + (dot[2] + dot[3]);
            if (scores_out != nullptr) scores_out[orow * shp.t_capacity + len + j0 + lane] = s;
        }
        const float m_new = fmaxf(m_run, wave_max(s));
        const float alpha = exp2_raw((m_run - m_new) * kLog2e);
        const float p = (lane < nj) ? exp2_raw((s - m_new) * kLog2e) : 0.0f;
        m_run = m_new;
        l_run = fmaf(l_run, alpha, wave_sum(p));
#pragma unroll
        for (int c = 0; c < CPT; ++c) acc[c] *= alpha;
        // eight value rows in flight; rows past the chunk's end are re-reads of its last row with weight zero
        for (int jb = 0; jb < nj; jb += 8) {
            float x[8][CPT];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int c = 0; c < CPT; ++c)
                    x[u][c] = load(v, v_is_bf16, v_row(j0 + min(jb + u, nj - 1)) * D + c * kWave + lane);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float pj = __shfl(p, min(jb + u, kWave - 1), kWave);   // p is zero in lanes >= nj
                const float wj = (jb + u < nj) ? pj : 0.0f;
#pragma unroll
                for (int c = 0; c < CPT; ++c) acc[c] = fmaf(wj, x[u][c], acc[c]);
            }
        }
    }
    if (lane == 0) {
        win_ml[orow * 2] = m_run;
        win_ml[orow * 2 + 1] = l_run;
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c) win_acc[orow * D + c * kWave + lane] = acc[c];
}

}  // namespace octopus

#endif
