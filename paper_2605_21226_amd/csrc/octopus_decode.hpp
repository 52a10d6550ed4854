// Fused decode attention over compressed keys (Alg. 2, Eq. (score-exact)): query rotation,
// split-K main kernel, split merge.
#ifndef OCTOPUS_DECODE_HPP_
#define OCTOPUS_DECODE_HPP_

#include "octopus_device.hpp"

namespace octopus {

constexpr float kLog2e = 1.4426950408889634f;

// ---- D0: q_rot = scale * H (s . q), one wavefront per query row ------------------------------
// Output layout per (sequence, KV head, row group): [QS coordinates][RG rows], so that the RG
// values a key needs for one coordinate are adjacent.  Rows past rows_per_kv and coordinates
// past d are written as zeros.
template <int D, int QS>
__global__ __launch_bounds__(kWave) void rotate_queries_kernel(const void *__restrict__ q, int q_is_bf16,
                                                                const uint8_t *__restrict__ signs, DecodeShape s,
                                                                float scale, float *__restrict__ q_rot) {
    constexpr int EPL = D / kWave;  // elements per lane (1, 2, 4)
    const int lane = threadIdx.x;
    const int rg = s.rows_per_pass;
    const int padded_rows = s.n_row_groups * rg;
    const int64_t gid = blockIdx.x;  // (seq, kvh, padded row)
    const int row = static_cast<int>(gid % padded_rows);
    const int kvh = static_cast<int>((gid / padded_rows) % s.n_kv_heads);
    const int seq = static_cast<int>(gid / (static_cast<int64_t>(padded_rows) * s.n_kv_heads));
    float *dst = q_rot + (gid / rg) * (static_cast<int64_t>(QS) * rg) + (row % rg);

    float x[EPL];
    if (row < s.rows_per_kv) {
        const int qi = row / s.heads_per_kv;
        const int head = kvh * s.heads_per_kv + row % s.heads_per_kv;
        const int64_t base = ((static_cast<int64_t>(seq) * s.n_q + qi) * s.n_q_heads + head) * D + lane * EPL;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int e = lane * EPL + j;
            float val = q_is_bf16 ? __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(q)[base + j]) << 16)
                                  : static_cast<const float *>(q)[base + j];
            const bool neg = (signs[kvh * (D / 8) + (e >> 3)] >> (e & 7)) & 1;
            x[j] = neg ? -val : val;
        }
        // butterflies over the in-lane bits of the element index ...
#pragma unroll
        for (int h = 1; h < EPL; h <<= 1) {
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                if ((j & h) == 0) {
                    const float a = x[j], b = x[j | h];
                    x[j] = a + b;
                    x[j | h] = a - b;
                }
            }
        }
        // ... then over the lane bits: the element with the bit clear takes a + b, the other a - b
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) {
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const float other = __shfl_xor(x[j], m, kWave);
                x[j] = (lane & m) ? other - x[j] : x[j] + other;
            }
        }
        const float norm = scale * (D == 64 ? 0.125f : (D == 128 ? 0.08838834764831845f : 0.0625f));
#pragma unroll
        for (int j = 0; j < EPL; ++j) x[j] *= norm;
    } else {
#pragma unroll
        for (int j = 0; j < EPL; ++j) x[j] = 0.0f;
    }
#pragma unroll
    for (int j = 0; j < EPL; ++j) dst[static_cast<int64_t>(lane * EPL + j) * rg] = x[j];
    for (int e = D + lane; e < QS; e += kWave) dst[static_cast<int64_t>(e) * rg] = 0.0f;
}

// ---- D1-D7: split-K main kernels --------------------------------------------------------------
// One workgroup of 4 wavefronts per (split, KV head x row group, sequence).  Each wavefront takes
// 64-token tiles of the split round-robin with one key per lane: the lane loads its record (16
// bytes at a time, coalesced thanks to the tile-interleaved layout), unpacks the code fields with
// compile-time shifts, looks the direction up in an LDS table and accumulates the RG scores against
// the wave-uniform rotated queries.  Wave results are merged in LDS and one partial (m, l, acc) is
// written per row.  Two variants differ in P.V only: decode_kernel_valu (fp32 values) sends the
// probabilities through LDS to a channel-per-lane mapping and multiplies on the vector ALUs;
// decode_kernel_mfma (bf16 values) feeds them to the matrix cores.
template <class P, int RG>
struct DecodeSmem {
    float4 lut0[P::LUT0];
    float4 lut1[P::LUT1 > 0 ? P::LUT1 : 1];
    float c_xi[2][32];
    float rho[2][8];
    float pbuf[4][kWave][RG];         // probabilities of the current tile, per wave
    float wave_m[4][RG], wave_l[4][RG];
    float red[4][RG][P::D];           // per-wave accumulators for the final merge
};

template <class P, int RG>
__device__ __forceinline__ void tile_scores(const uint32_t (&w)[P::NWORDS], const float *__restrict__ qg,
                                            const DecodeSmem<P, RG> &sm, float (&s)[RG]) {
#pragma unroll
    for (int r = 0; r < RG; ++r) s[r] = 0.0f;
    static_for<0, P::NTRI>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int c = P::cls(i);
        const uint32_t code = field<P::dir_bit(i), 2 * P::bdir(i)>(w);
        const uint32_t ridx = field<P::nrm_bit(i), P::bnrm(i)>(w);
        const float4 n = c ? sm.lut1[code] : sm.lut0[code];
        const float rho = sm.rho[c][ridx];
        const float tx = rho * n.x, ty = rho * n.y, tz = rho * n.z;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            s[r] = fmaf(qg[(3 * i) * RG + r], tx, s[r]);
            s[r] = fmaf(qg[(3 * i + 1) * RG + r], ty, s[r]);
            s[r] = fmaf(qg[(3 * i + 2) * RG + r], tz, s[r]);  // rotated queries are zero past d
        }
    });
}

template <class P, int RG>
__global__ __launch_bounds__(256) void decode_kernel_valu(DeviceBooks books, DecodeShape shp,
                                                      const float *__restrict__ q_rot,
                                                      const uint4 *__restrict__ cache, const void *__restrict__ v,
                                                      int v_is_bf16, const int32_t *__restrict__ seq_lens,
                                                      float *__restrict__ part_ml, float *__restrict__ part_acc,
                                                      float *__restrict__ scores_out) {
    constexpr int D = P::D;
    constexpr int LPR = D / 8;          // lanes per V row (8 channels per lane)
    constexpr int KPL = kWave / LPR;    // V rows per wave-wide load
    __shared__ DecodeSmem<P, RG> sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x;
    const int kvh = blockIdx.y / shp.n_row_groups, grp = blockIdx.y % shp.n_row_groups;
    const int seq = blockIdx.z;
    const int len = seq_lens[seq];
    const int t_begin = split * shp.split_len;
    if (t_begin >= len) return;  // the merge only reads splits that start below len
    const int t_end = min(len, t_begin + shp.split_len);

    if (wave == 0) copy_books(books, sm.c_xi, sm.rho);
    __syncthreads();
    build_dir_lut<P::BD0>(sm.lut0, sm.c_xi[0], tid, 256);
    if constexpr (P::NCLASS == 2) build_dir_lut<P::BD1>(sm.lut1, sm.c_xi[1], tid, 256);
    __syncthreads();

    const int64_t pair = static_cast<int64_t>(seq) * shp.n_kv_heads + kvh;
    const int64_t group_id = pair * shp.n_row_groups + grp;
    const float *qg = q_rot + group_id * (P::QS * RG);
    const uint4 *region = cache + pair * (shp.t_capacity * P::GRANULES);
    const int64_t v_row0 = pair * shp.t_capacity;

    float m_run[RG], l_lane[RG], acc[RG][8];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        m_run[r] = -INFINITY;
        l_lane[r] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[r][c] = 0.0f;
    }
    const int rl = lane % LPR, ko = lane / LPR;

    for (int t0 = t_begin + wave * kWave; t0 < t_end; t0 += 4 * kWave) {
        // D1: this lane's record
        uint32_t w[P::NWORDS];
        const uint4 *tile = region + static_cast<int64_t>(t0 / kWave) * (P::GRANULES * kWave) + lane;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            const uint4 x = tile[g * kWave];
            w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = x.w;
        }
        // D2-D4: scores (queries carry the softmax scale already)
        float s[RG];
        tile_scores<P, RG>(w, qg, sm, s);
        const float gamma = __uint_as_float(w[0]);
        const bool valid = (t0 + lane) < t_end;
#pragma unroll
        for (int r = 0; r < RG; ++r) s[r] = valid ? s[r] * gamma : -INFINITY;
        if (scores_out != nullptr && valid) {
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int row = grp * RG + r;
                if (row < shp.rows_per_kv) {
                    const int qi = row / shp.heads_per_kv, head = kvh * shp.heads_per_kv + row % shp.heads_per_kv;
                    scores_out[((static_cast<int64_t>(seq) * shp.n_q + qi) * shp.n_q_heads + head) * shp.t_capacity +
                               t0 + lane] = s[r];
                }
            }
        }
        // D5: online softmax, one running maximum per row for the whole wave
        float alpha[RG];
        bool rescale = false;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const float m_new = fmaxf(m_run[r], wave_max(s[r]));
            alpha[r] = exp2f((m_run[r] - m_new) * kLog2e);
            rescale |= (m_new != m_run[r]);
            m_run[r] = m_new;
            const float p = exp2f((s[r] - m_new) * kLog2e);
            l_lane[r] = l_lane[r] * alpha[r] + p;
            sm.pbuf[wave][lane][r] = p;
        }
        if (rescale) {
#pragma unroll
            for (int r = 0; r < RG; ++r)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[r][c] *= alpha[r];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // D6: P.V with 8 channels per lane; lanes with the same ko walk the same keys
        const int n_valid = min(kWave, t_end - t0);
        for (int kb = 0; kb < n_valid; kb += KPL) {
            const int key = kb + ko;
            float pv[RG];
#pragma unroll
            for (int r = 0; r < RG; ++r) pv[r] = sm.pbuf[wave][key][r];
            float vals[8];
            const int64_t vrow = v_row0 + t0 + key;
            if (key < n_valid) {
                if (v_is_bf16) {
                    const uint4 x = static_cast<const uint4 *>(v)[vrow * (D / 8) + rl];
                    vals[0] = bf16_lo(x.x); vals[1] = bf16_hi(x.x); vals[2] = bf16_lo(x.y); vals[3] = bf16_hi(x.y);
                    vals[4] = bf16_lo(x.z); vals[5] = bf16_hi(x.z); vals[6] = bf16_lo(x.w); vals[7] = bf16_hi(x.w);
                } else {
                    const float4 a = static_cast<const float4 *>(v)[vrow * (D / 4) + 2 * rl];
                    const float4 b = static_cast<const float4 *>(v)[vrow * (D / 4) + 2 * rl + 1];
                    vals[0] = a.x; vals[1] = a.y; vals[2] = a.z; vals[3] = a.w;
                    vals[4] = b.x; vals[5] = b.y; vals[6] = b.z; vals[7] = b.w;
                }
#pragma unroll
                for (int r = 0; r < RG; ++r)
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[r][c] = fmaf(pv[r], vals[c], acc[r][c]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // D7: fold the KPL lane groups, then the 4 wavefronts, and emit one partial per row
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1)
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] += __shfl_xor(acc[r][c], o, kWave);
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const float l = wave_sum(l_lane[r]);
        if (lane == 0) { sm.wave_m[wave][r] = m_run[r]; sm.wave_l[wave][r] = l; }
        if (ko == 0) {
#pragma unroll
            for (int c = 0; c < 8; ++c) sm.red[wave][r][rl * 8 + c] = acc[r][c];
        }
    }
    __syncthreads();
    for (int e = tid; e < RG * D; e += 256) {
        const int r = e / D, c = e % D;
        const int row = grp * RG + r;
        if (row >= shp.rows_per_kv) continue;
        float m = sm.wave_m[0][r];
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) m = fmaxf(m, sm.wave_m[wv][r]);
        float l = 0.0f, a = 0.0f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float mw = sm.wave_m[wv][r];
            const float f = (mw == -INFINITY) ? 0.0f : exp2f((mw - m) * kLog2e);
            l += f * sm.wave_l[wv][r];
            a += f * sm.red[wv][r][c];
        }
        const int64_t prow = (group_id * RG + r) * shp.n_splits + split;
        part_acc[prow * D + c] = a;
        if (c == 0) { part_ml[prow * 2] = m; part_ml[prow * 2 + 1] = l; }
    }
}


// ---- bf16 values: P.V on the matrix cores -------------------------------------------------------
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] B[32x16]; lane l holds row l%16 of A and
// column l%16 of B, each for the 8 k-slots of lane group l/16, and rows 4*(l/16)..+3 of column l%16
// of D.  Here M = probability rows, K = keys, N = channels:
//   * a 64-key tile is two k-steps; k-slot (g, j) of step ks is key 32*ks + 4*j + g, so that one
//     wave-wide value load (fixed j) reads 4 consecutive value rows;
//   * lane (n, g) loads CPL = d/16 adjacent channels [CPL*n, CPL*n + CPL) of its 8 keys per k-step;
//     N-block c of the MFMA is the channel set {CPL*n + c}, so B operands are byte permutes of the
//     loaded registers and values are never converted;
//   * a probability is split into two bf16 numbers, hi = its upper 16 bits and lo = the rest, which
//     occupy rows r and RP + r of A; the two partial results are added at the end.  The relative
//     error of hi + lo is below 2^-16.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kPRow = 72;  // bf16 per probability row in LDS: 64 keys + 8 pad (144-byte stride)

template <class P, int RG>
struct DecodeSmemMfma {
    float4 lut0[P::LUT0];
    float4 lut1[P::LUT1 > 0 ? P::LUT1 : 1];
    float c_xi[2][32];
    float rho[2][8];
    uint16_t pbuf[4][16][kPRow];
    float wave_m[4][RG], wave_l[4][RG];
    float red[4][RG][P::D];
};

template <class P, int RG, class SM>
__device__ __forceinline__ void tile_scores_t(const uint32_t (&w)[P::NWORDS], const float *__restrict__ qg,
                                              const SM &sm, float (&s)[RG]) {
#pragma unroll
    for (int r = 0; r < RG; ++r) s[r] = 0.0f;
    static_for<0, P::NTRI>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int c = P::cls(i);
        const uint32_t code = field<P::dir_bit(i), 2 * P::bdir(i)>(w);
        const uint32_t ridx = field<P::nrm_bit(i), P::bnrm(i)>(w);
        const float4 n = c ? sm.lut1[code] : sm.lut0[code];
        const float rho = sm.rho[c][ridx];
        const float tx = rho * n.x, ty = rho * n.y, tz = rho * n.z;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            s[r] = fmaf(qg[(3 * i) * RG + r], tx, s[r]);
            s[r] = fmaf(qg[(3 * i + 1) * RG + r], ty, s[r]);
            s[r] = fmaf(qg[(3 * i + 2) * RG + r], tz, s[r]);  // rotated queries are zero past d
        }
    });
}

template <class P, int RG>
__global__ __launch_bounds__(256) void decode_kernel_mfma(DeviceBooks books, DecodeShape shp,
                                                           const float *__restrict__ q_rot,
                                                           const uint4 *__restrict__ cache,
                                                           const uint32_t *__restrict__ v,
                                                           const int32_t *__restrict__ seq_lens,
                                                           float *__restrict__ part_ml, float *__restrict__ part_acc,
                                                           float *__restrict__ scores_out) {
    constexpr int D = P::D;
    constexpr int CPL = D / 16;            // channels per lane chunk = N-blocks
    constexpr int CW = CPL / 2;            // 32-bit words per chunk
    constexpr int RP = RG < 4 ? 4 : RG;    // probability rows padded to a multiple of 4
    __shared__ DecodeSmemMfma<P, RG> sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x;
    const int kvh = blockIdx.y / shp.n_row_groups, grp = blockIdx.y % shp.n_row_groups;
    const int seq = blockIdx.z;
    const int len = seq_lens[seq];
    const int t_begin = split * shp.split_len;
    if (t_begin >= len) return;  // the merge only reads splits that start below len
    const int t_end = min(len, t_begin + shp.split_len);

    if (wave == 0) copy_books(books, sm.c_xi, sm.rho);
    for (int e = tid; e < 4 * 16 * kPRow; e += 256) (&sm.pbuf[0][0][0])[e] = 0;
    __syncthreads();
    build_dir_lut<P::BD0>(sm.lut0, sm.c_xi[0], tid, 256);
    if constexpr (P::NCLASS == 2) build_dir_lut<P::BD1>(sm.lut1, sm.c_xi[1], tid, 256);
    __syncthreads();

    const int64_t pair = static_cast<int64_t>(seq) * shp.n_kv_heads + kvh;
    const int64_t group_id = pair * shp.n_row_groups + grp;
    const float *qg = q_rot + group_id * (P::QS * RG);
    const uint4 *region = cache + pair * (shp.t_capacity * P::GRANULES);
    const int n16 = lane & 15, g4 = lane >> 4;
    // value words of this lane: row stride D/2 words, chunk at word CW * n16
    const uint32_t *v_lane = v + pair * shp.t_capacity * (D / 2) + CW * n16;
    const int ppos = (lane & 32) + 8 * (lane & 3) + ((lane & 31) >> 2);  // slot of key `lane` in a pbuf row

    float m_run[RG], l_lane[RG];
    f32x4_t acc[CPL];
#pragma unroll
    for (int r = 0; r < RG; ++r) { m_run[r] = -INFINITY; l_lane[r] = 0.0f; }
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

    for (int t0 = t_begin + wave * kWave; t0 < t_end; t0 += 4 * kWave) {
        const int n_valid = min(kWave, t_end - t0);
        // D6 operands first, so that they are in flight during the score phase: 8 keys x CPL channels
        // per k-step and lane
        uint32_t vr[2][8][CW];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = 32 * ks + 4 * j + g4;
                const uint32_t *src = v_lane + static_cast<int64_t>(t0 + key) * (D / 2);
                if (n_valid == kWave || key < n_valid) {
                    if constexpr (CW == 2) {
                        const uint2 x = *reinterpret_cast<const uint2 *>(src);
                        vr[ks][j][0] = x.x; vr[ks][j][1] = x.y;
                    } else {
#pragma unroll
                        for (int q4 = 0; q4 < CW / 4; ++q4) {
                            const uint4 x = reinterpret_cast<const uint4 *>(src)[q4];
                            vr[ks][j][4 * q4] = x.x; vr[ks][j][4 * q4 + 1] = x.y;
                            vr[ks][j][4 * q4 + 2] = x.z; vr[ks][j][4 * q4 + 3] = x.w;
                        }
                    }
                } else {
#pragma unroll
                    for (int cw = 0; cw < CW; ++cw) vr[ks][j][cw] = 0u;
                }
            }
        // D1: this lane's record
        uint32_t w[P::NWORDS];
        const uint4 *tile = region + static_cast<int64_t>(t0 / kWave) * (P::GRANULES * kWave) + lane;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            const uint4 x = tile[g * kWave];
            w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = x.w;
        }
        // D2-D4: scores (queries carry the softmax scale already)
        float s[RG];
        tile_scores_t<P, RG>(w, qg, sm, s);
        const float gamma = __uint_as_float(w[0]);
        const bool valid = lane < n_valid;
#pragma unroll
        for (int r = 0; r < RG; ++r) s[r] = valid ? s[r] * gamma : -INFINITY;
        if (scores_out != nullptr && valid) {
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int row = grp * RG + r;
                if (row < shp.rows_per_kv) {
                    const int qi = row / shp.heads_per_kv, head = kvh * shp.heads_per_kv + row % shp.heads_per_kv;
                    scores_out[((static_cast<int64_t>(seq) * shp.n_q + qi) * shp.n_q_heads + head) * shp.t_capacity +
                               t0 + lane] = s[r];
                }
            }
        }
        // D5: online softmax, one running maximum per row for the whole wave
        float alpha[RG];
        bool rescale = false;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const float m_new = fmaxf(m_run[r], wave_max(s[r]));
            alpha[r] = exp2f((m_run[r] - m_new) * kLog2e);
            rescale |= (m_new != m_run[r]);
            m_run[r] = m_new;
            const float p = exp2f((s[r] - m_new) * kLog2e);
            l_lane[r] = fmaf(l_lane[r], alpha[r], p);
            const uint32_t pb = __float_as_uint(p);
            const float lo = p - __uint_as_float(pb & 0xffff0000u);
            sm.pbuf[wave][r][ppos] = static_cast<uint16_t>(pb >> 16);
            sm.pbuf[wave][RP + r][ppos] = static_cast<uint16_t>(__float_as_uint(lo) >> 16);
        }
        if (rescale) {
            // accumulator rows of this lane: m = 4 * g4 + i, probability row r = m % RP
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float a;
                if constexpr (RP == 4) {
                    a = i < RG ? alpha[i < RG ? i : 0] : 1.0f;
                } else {
                    a = (g4 & 1) ? alpha[4 + i] : alpha[i];
                }
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c][i] *= a;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // D6: P.V
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            union { uint4 u; bf16x8_t b; } pa;
            pa.u = *reinterpret_cast<const uint4 *>(&sm.pbuf[wave][n16][32 * ks + 8 * g4]);
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                union { uint32_t u[4]; bf16x8_t b; } vb;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    vb.u[jj] = __builtin_amdgcn_perm(vr[ks][2 * jj + 1][c / 2], vr[ks][2 * jj][c / 2],
                                                     (c & 1) ? 0x07060302u : 0x05040100u);
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.b, vb.b, acc[c], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // D7: add the hi and lo partial results (lane groups RP/4 apart), then fold the 4 wavefronts
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float tot = acc[c][i] + __shfl_down(acc[c][i], RP * 4, kWave);
            const int r = 4 * g4 + i;
            if (r < RG) sm.red[wave][r][CPL * n16 + c] = tot;
        }
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const float l = wave_sum(l_lane[r]);
        if (lane == 0) { sm.wave_m[wave][r] = m_run[r]; sm.wave_l[wave][r] = l; }
    }
    __syncthreads();
    for (int e = tid; e < RG * D; e += 256) {
        const int r = e / D, c = e % D;
        const int row = grp * RG + r;
        if (row >= shp.rows_per_kv) continue;
        float m = sm.wave_m[0][r];
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) m = fmaxf(m, sm.wave_m[wv][r]);
        float l = 0.0f, a = 0.0f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float mw = sm.wave_m[wv][r];
            const float f = (mw == -INFINITY) ? 0.0f : exp2f((mw - m) * kLog2e);
            l += f * sm.wave_l[wv][r];
            a += f * sm.red[wv][r][c];
        }
        const int64_t prow = (group_id * RG + r) * shp.n_splits + split;
        part_acc[prow * D + c] = a;
        if (c == 0) { part_ml[prow * 2] = m; part_ml[prow * 2 + 1] = l; }
    }
}

// ---- D8: merge of the split partials ----------------------------------------------------------
template <int D>
__global__ __launch_bounds__(D) void merge_kernel(DecodeShape shp, const int32_t *__restrict__ seq_lens,
                                                   const float *__restrict__ part_ml,
                                                   const float *__restrict__ part_acc, float *__restrict__ out) {
    const int c = threadIdx.x;
    const int64_t orow = blockIdx.x;  // (seq, qi, head)
    const int head = static_cast<int>(orow % shp.n_q_heads);
    const int qi = static_cast<int>((orow / shp.n_q_heads) % shp.n_q);
    const int seq = static_cast<int>(orow / (static_cast<int64_t>(shp.n_q_heads) * shp.n_q));
    const int kvh = head / shp.heads_per_kv;
    const int row = qi * shp.heads_per_kv + head % shp.heads_per_kv;
    const int grp = row / shp.rows_per_pass, r = row % shp.rows_per_pass;
    const int64_t prow0 =
        (((static_cast<int64_t>(seq) * shp.n_kv_heads + kvh) * shp.n_row_groups + grp) * shp.rows_per_pass + r) *
        shp.n_splits;
    const int len = seq_lens[seq];
    const int n_valid = min((len + shp.split_len - 1) / shp.split_len, shp.n_splits);  // splits that start below len
    float m = -INFINITY;
    for (int j = 0; j < n_valid; ++j) m = fmaxf(m, part_ml[(prow0 + j) * 2]);
    float l = 0.0f, a = 0.0f;
    for (int j = 0; j < n_valid; ++j) {
        const float f = exp2f((part_ml[(prow0 + j) * 2] - m) * kLog2e);
        l += f * part_ml[(prow0 + j) * 2 + 1];
        a += f * part_acc[(prow0 + j) * D + c];
    }
    out[orow * D + c] = n_valid > 0 ? a / l : 0.0f;
}

// ---- launch helpers -----------------------------------------------------------------------------
template <class P, int RG>
int launch_decode_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                     const void *v, int v_dtype, const int32_t *seq_lens, float *part_ml, float *part_acc,
                     float *scores_out, hipStream_t stream) {
    DeviceBooks books;
    for (int c = 0; c < 2; ++c) {
        for (int k = 0; k < 32; ++k) books.c_xi[c][k] = cb.c_xi[c][k];
        for (int k = 0; k < 8; ++k) books.c_rho[c][k] = cb.c_rho[c][k];
    }
    const dim3 grid(s.n_splits, s.n_kv_heads * s.n_row_groups, s.n_seq);
    if (v_dtype == OCTOPUS_DTYPE_BF16)
        hipLaunchKernelGGL((decode_kernel_mfma<P, RG>), grid, dim3(256), 0, stream, books, s, q_rot,
                           static_cast<const uint4 *>(cache), static_cast<const uint32_t *>(v), seq_lens, part_ml,
                           part_acc, scores_out);
    else
        hipLaunchKernelGGL((decode_kernel_valu<P, RG>), grid, dim3(256), 0, stream, books, s, q_rot,
                           static_cast<const uint4 *>(cache), v, 0, seq_lens, part_ml, part_acc, scores_out);
    return static_cast<int>(hipGetLastError());
}

template <class P>
int launch_decode_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                       const void *v, int v_dtype, const int32_t *seq_lens, float *part_ml, float *part_acc,
                       float *scores_out, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_rg<P, 1>(cb, s, q_rot, cache, v, v_dtype, seq_lens, part_ml, part_acc, scores_out, stream);
        case 2: return launch_decode_rg<P, 2>(cb, s, q_rot, cache, v, v_dtype, seq_lens, part_ml, part_acc, scores_out, stream);
        case 4: return launch_decode_rg<P, 4>(cb, s, q_rot, cache, v, v_dtype, seq_lens, part_ml, part_acc, scores_out, stream);
        case 8: return launch_decode_rg<P, 8>(cb, s, q_rot, cache, v, v_dtype, seq_lens, part_ml, part_acc, scores_out, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace octopus

#endif
