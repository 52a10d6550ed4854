// Decode attention for many query rows per KV head (a chunk of queries against the whole cache, e.g. the
// 3600 queries of a video frame): Alg. 2 with the roles of a dense attention kernel.  Here the work per
// key is a dense contraction over hundreds of rows, so both products run on the matrix cores; the keys
// are still decoded on the fly from the packed records, once per 128 query rows, into an LDS tile and
// never reach memory.
//
// A workgroup of 4 wavefronts owns 128 query rows of one (sequence, KV head) (32 per wavefront) and a
// range of 64-token tiles.  Per tile:
//   * stage (all 256 threads, one tile ahead, double-buffered LDS): lane = key; the record is unpacked,
//     gamma * rho^ * n^ is looked up and multiplied, split into two bf16 numbers (hi = upper 16 bits,
//     lo = the rest) and written to the key tile [key][coordinate]; the values of the tile are written
//     transposed [channel][key];
//   * S^T = K^ Q^T (keys x rows) with v_mfma_f32_32x32x16_bf16, three products per k-step (hi hi, hi lo,
//     lo hi: relative error below 2^-16); a lane then holds 32 scores of ONE query row, so the softmax
//     statistics of a row live in one lane (and its partner lane + 32);
//   * O^T += V^T P^T (channels x rows): the probabilities go from the accumulators of the first product
//     straight into the B operand of the second (k-slot j of lane group h is key 4h + j, or 8 + 4h + j - 4
//     for j >= 4, of each group of 16 keys, which is how the first product left them), again as hi + lo.
// The partial (m, l, acc) of each row goes to the split-K workspace and through the same merge kernel as
// the single-query path.
#ifndef OCTOPUS_DECODE_MQ_HPP_
#define OCTOPUS_DECODE_MQ_HPP_

#include "octopus_decode.hpp"

namespace octopus {

// Query rows per workgroup: 32 per wavefront, NW = 4 wavefronts (128 rows) or, at d = 64 where the
// registers allow two wavefronts per SIMD, NW = 8 (256 rows).  The keys of a tile are decoded once per
// workgroup, so more rows mean less decoding; the host picks 256 when there are rows enough to fill them.

typedef __attribute__((ext_vector_type(16))) float f32x16_t;
constexpr int kXcds = 8;   // accelerator dies of the chip; consecutive workgroups go to consecutive dies

template <class P>
struct MqSmem {
    static constexpr int D = P::D;
    static constexpr int KST = D + 8;       // bf16 per row of the key tile: 16-byte reads of 8 lanes hit 8 bank groups
    static constexpr int VST = kWave + 4;   // bf16 per row of the transposed value tile (8-byte aligned rows)
    float4 dir0[1 << (2 * P::BD0)];
    float4 dir1[P::NCLASS == 2 ? 1 << (2 * P::BD1) : 1];
    float c_xi[2][kMaxLevels];
    float c_rho[2][kMaxLevels];
    uint16_t kh[2][kWave][KST];
    uint16_t kl[2][kWave][KST];
    uint16_t vt[2][D][VST];
};

template <class P, int NW>
__global__ __launch_bounds__(kWave *NW) __attribute__((amdgpu_waves_per_eu(P::D <= 64 ? 2 : 1))) void decode_kernel_mq(DeviceBooks books, DecodeShape shp,
                                                         const float *__restrict__ q_rot,
                                                         const uint4 *__restrict__ cache,
                                                         const uint16_t *__restrict__ v,
                                                         const int32_t *__restrict__ seq_lens,
                                                         float *__restrict__ part_ml, float *__restrict__ part_acc,
                                                         PageTable pt) {
    // pt.table (or NULL): `cache` and `v` are pools of 64-token pages, [page][KV head] each a key tile and 64 value
    // rows; logical tile j of sequence s lives in page pt.table[s * pt.stride + j] (clamped to the pool)
    constexpr int D = P::D;
    constexpr int KK = D / 16;               // k-steps of the score product
    constexpr int NB = D / 32;               // 32-channel blocks of the output
    constexpr int ROWB = D * 2;              // bytes per value row
    constexpr int TILEB = P::GRANULES * kWave * 16;
    constexpr int ROWS = 32 * NW;            // query rows per workgroup
    constexpr int VP = D / 8 / NW;           // 16-byte value pieces per thread and tile
    using S = MqSmem<P>;
    __shared__ S sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;

    // tables (one copy: the lookups are a small part of this kernel)
    if (tid < kWave) copy_books<P>(books, sm.c_xi, sm.c_rho);
    __syncthreads();
    build_dir_lut<P::BD0>(sm.dir0, sm.c_xi[0], tid, kWave * NW);
    if constexpr (P::NCLASS == 2) build_dir_lut<P::BD1>(sm.dir1, sm.c_xi[1], tid, kWave * NW);

    // work: (sequence, KV head, block of ROWS rows, split) and the split's tiles.  The blocks of rows of one
    // (sequence, KV head, split) read the same keys and values: they are given to ONE accelerator die (workgroup
    // b runs on die b % 8, each with its own L2), next to each other in that die's sequence of workgroups, so
    // that the tiles are fetched from memory once and not once per die.  Unit u = (pair, split) goes to die
    // u % 8; the grid is padded to whole rounds of 8 units (the workgroups of units that do not exist leave).
    const int64_t slot = blockIdx.x / kXcds;
    const int64_t unit = (slot / shp.n_row_groups) * kXcds + blockIdx.x % kXcds;
    const int64_t n_units = static_cast<int64_t>(shp.n_seq) * shp.n_kv_heads * shp.n_splits;
    if (unit >= n_units) return;   // (whole workgroup, before any barrier)
    const int split = static_cast<int>(unit % shp.n_splits);
    const int64_t pair = unit / shp.n_splits;
    const int64_t group_id = pair * shp.n_row_groups + slot % shp.n_row_groups;
    const int seq = static_cast<int>(pair / shp.n_kv_heads);
    const int len = min(max(seq_lens[seq], 0), shp.max_len);
    const int n_tiles = (len + kWave - 1) / kWave;
    const int base = n_tiles / shp.n_splits, rem = n_tiles % shp.n_splits;
    const int tile_begin = split * base + min(split, rem);
    const int tile_end = tile_begin + base + (split < rem ? 1 : 0);

    const bool paged = pt.table != nullptr;
    const int kvh = static_cast<int>(pair % shp.n_kv_heads);
    const char *k_region = reinterpret_cast<const char *>(cache) + (paged ? 0 : pair * shp.t_capacity * (P::GRANULES * 16));
    const char *v_pair = reinterpret_cast<const char *>(v) + (paged ? 0 : pair * shp.t_capacity * ROWB);

    // Q^T operands of this wave's 32 rows: lane (n, h) holds coordinates 16 kk + 8 h .. + 8 of row n as
    // bf16 hi and lo.  The rotated queries lie [coordinate][row] with the ROWS rows of the block adjacent.
    const float *qg = q_rot + group_id * (static_cast<int64_t>(P::QS) * ROWS) + wave * 32 + n;
    union BF8 { uint32_t u[4]; bf16x8_t b; };
    BF8 qh[KK], ql[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = qg[(16 * kk + 8 * h + 2 * e) * ROWS], b = qg[(16 * kk + 8 * h + 2 * e + 1) * ROWS];
            const uint32_t ab = __float_as_uint(a), bb = __float_as_uint(b);
            qh[kk].u[e] = __builtin_amdgcn_perm(bb, ab, 0x07060302u);
            const float al = a - __uint_as_float(ab & 0xffff0000u), bl = b - __uint_as_float(bb & 0xffff0000u);
            ql[kk].u[e] = __builtin_amdgcn_perm(__float_as_uint(bl), __float_as_uint(al), 0x07060302u);
        }

    // ---- staging: global -> registers -> LDS tile ---------------------------------------------------
    uint32_t w[P::NWORDS];          // this lane's record of the tile being staged
    uint4 vp[VP];                   // its value pieces: key `lane`, channels 8 (wave + 4 i) .. + 8
    auto load_tile = [&](int tile) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));
        constexpr int USED = (P::RECORD_BYTES + 3) / 4;
        // position of the tile in the cache (in tiles): the logical tile, or its page's tile of this KV head
        int64_t slot = tile;
        if (paged) {
            const int page = pt.table[static_cast<int64_t>(seq) * pt.stride + tile];
            slot = static_cast<int64_t>(min(max(page, 0), pt.n_pages - 1)) * shp.n_kv_heads + kvh;
        }
        const char *src = k_region + slot * TILEB + lane * 16;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            const char *gp = src + g * (kWave * 16);
            const int nw = (USED - 4 * g) < 4 ? (USED - 4 * g) : 4;
            if (nw == 4) {
                const uint4 x = *reinterpret_cast<const uint4 *>(gp);
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = x.w;
            } else if (nw == 3) {
                const u32x3_t x = *reinterpret_cast<const u32x3_t *>(gp);
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = 0u;
            } else if (nw == 2) {
                const u32x2_t x = *reinterpret_cast<const u32x2_t *>(gp);
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = 0u; w[4 * g + 3] = 0u;
            } else {
                w[4 * g] = *reinterpret_cast<const uint32_t *>(gp);
                w[4 * g + 1] = 0u; w[4 * g + 2] = 0u; w[4 * g + 3] = 0u;
            }
        }
        // value rows past the sequence's end are replaced by its last row (their probabilities are zero)
        // (that row is in the same tile, hence in the same page)
        const int row = min(tile * kWave + lane, len - 1);
        const char *vrow = v_pair + (slot * kWave + (row - tile * kWave)) * ROWB;
#pragma unroll
        for (int i = 0; i < VP; ++i) vp[i] = *reinterpret_cast<const uint4 *>(vrow + (wave + NW * i) * 16);
    };
    // Wave wv writes the coordinates [wv * D / NW, (wv + 1) * D / NW) of its lane's key: it decodes the triplets
    // that cover them (one or two of them are decoded by the neighbouring wave as well) and writes whole
    // 16-byte pieces of the key tile.  (Two-byte writes, one per coordinate, land on 8 banks for the 64 lanes
    // of a wavefront and were a third of this kernel's time.)
    auto stage_block = [&](auto ww, int buf) __attribute__((always_inline)) {
        constexpr int wv = decltype(ww)::value;
        constexpr int CW = D / NW;                      // coordinates per wave: 8 (d = 64) or 32 (d = 128)
        constexpr int T_LO = (wv * CW) / 3, T_HI = ((wv + 1) * CW - 1) / 3;
        constexpr int NT = T_HI - T_LO + 1;
        float val[3 * NT];
        static_for<0, NT>([&](auto jj) {
            constexpr int i = T_LO + decltype(jj)::value;
            constexpr int c = P::cls(i);
            constexpr int bd = P::bdir(i), bn = P::bnrm(i);
            const uint32_t code = field<P::dir_bit(i), 2 * bd>(w);
            const uint32_t nrm = field<P::nrm_bit(i), bn>(w);
            const float4 dir = (c ? sm.dir1 : sm.dir0)[code];
            const float g = __uint_as_float(w[0]) * sm.c_rho[c][nrm];
            val[3 * decltype(jj)::value] = g * dir.x;
            val[3 * decltype(jj)::value + 1] = g * dir.y;
            val[3 * decltype(jj)::value + 2] = g * dir.z;
        });
#pragma unroll
        for (int g8 = 0; g8 < CW / 8; ++g8) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int j = wv * CW + 8 * g8 + 2 * k - 3 * T_LO;      // index into val of the pair's first value
                const uint32_t b0 = __float_as_uint(val[j]), b1 = __float_as_uint(val[j + 1]);
                const float l0 = val[j] - __uint_as_float(b0 & 0xffff0000u);
                const float l1 = val[j + 1] - __uint_as_float(b1 & 0xffff0000u);
                hi[k] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
                lo[k] = __builtin_amdgcn_perm(__float_as_uint(l1), __float_as_uint(l0), 0x07060302u);
            }
            *reinterpret_cast<uint4 *>(&sm.kh[buf][lane][wv * CW + 8 * g8]) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<uint4 *>(&sm.kl[buf][lane][wv * CW + 8 * g8]) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
    };
    auto stage_tile = [&](int buf) {
        switch (wave) {
            case 0: stage_block(std::integral_constant<int, 0>{}, buf); break;
            case 1: stage_block(std::integral_constant<int, 1>{}, buf); break;
            case 2: stage_block(std::integral_constant<int, 2>{}, buf); break;
            case 3: stage_block(std::integral_constant<int, 3>{}, buf); break;
            default:
                if constexpr (NW == 8) {
                    switch (wave) {
                        case 4: stage_block(std::integral_constant<int, 4>{}, buf); break;
                        case 5: stage_block(std::integral_constant<int, 5>{}, buf); break;
                        case 6: stage_block(std::integral_constant<int, 6>{}, buf); break;
                        default: stage_block(std::integral_constant<int, 7>{}, buf); break;
                    }
                }
                break;
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int c0 = (wave + NW * i) * 8;
            const uint32_t x[4] = {vp[i].x, vp[i].y, vp[i].z, vp[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sm.vt[buf][c0 + 2 * e][lane] = static_cast<uint16_t>(x[e] & 0xffffu);
                sm.vt[buf][c0 + 2 * e + 1][lane] = static_cast<uint16_t>(x[e] >> 16);
            }
        }
    };

    float m_run = -INFINITY, l_run = 0.0f;
    f32x16_t oacc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[nb][e] = 0.0f;

    if (tile_begin < tile_end) {
        load_tile(tile_begin);
        __syncthreads();                       // tables complete
        stage_tile(0);
        load_tile(min(tile_begin + 1, tile_end - 1));
    }
    __syncthreads();

    // With 8 wavefronts (two per SIMD: w and w + 4) the upper four stage the next tile BEFORE they work on
    // the current one, the lower four after: the two wavefronts of a SIMD are then in opposite phases, one
    // on the matrix cores while the other decodes keys on the vector units.
    const bool stage_first = NW == 8 && wave >= 4;
    for (int tile = tile_begin; tile < tile_end; ++tile) {
        const int buf = (tile - tile_begin) & 1;
        if (stage_first && tile + 1 < tile_end) {
            stage_tile(buf ^ 1);
            load_tile(min(tile + 2, tile_end - 1));
        }
        // S^T = K^ Q^T for the tile's two blocks of 32 keys
        f32x16_t sacc[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[mb][e] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                BF8 ah, al;
                *reinterpret_cast<uint4 *>(ah.u) = *reinterpret_cast<const uint4 *>(&sm.kh[buf][32 * mb + n][16 * kk + 8 * h]);
                *reinterpret_cast<uint4 *>(al.u) = *reinterpret_cast<const uint4 *>(&sm.kl[buf][32 * mb + n][16 * kk + 8 * h]);
                sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah.b, qh[kk].b, sacc[mb], 0, 0, 0);
                sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah.b, ql[kk].b, sacc[mb], 0, 0, 0);
                sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al.b, qh[kk].b, sacc[mb], 0, 0, 0);
            }
        }
        // keys past the end of the sequence (last tile only): element e of block mb is key
        // 32 mb + 8 (e / 4) + 4 h + e % 4
        const int n_valid = len - tile * kWave;
        if (n_valid < kWave) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (32 * mb + 8 * (e / 4) + 4 * h + (e % 4) >= n_valid) sacc[mb][e] = -INFINITY;
        }
        // online softmax of this lane's row (its other 32 keys of the tile are in lane + 32)
        float mx = sacc[0][0];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[mb][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2_raw((m_run - m_new) * kLog2e);
        m_run = m_new;
        const float m_log2 = -m_new * kLog2e;     // p = 2^(s log2(e) - m log2(e)): one fma per score
        float psum = 0.0f;
        BF8 ph[4], pl[4];   // per group of 16 keys: the 8 k-slots of this lane, hi and lo
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float p0 = exp2_raw(fmaf(sacc[mb][e], kLog2e, m_log2)), p1 = exp2_raw(fmaf(sacc[mb][e + 1], kLog2e, m_log2));
                psum += p0 + p1;
                const uint32_t b0 = __float_as_uint(p0), b1 = __float_as_uint(p1);
                const float l0 = p0 - __uint_as_float(b0 & 0xffff0000u), l1 = p1 - __uint_as_float(b1 & 0xffff0000u);
                ph[2 * mb + e / 8].u[(e % 8) / 2] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
                pl[2 * mb + e / 8].u[(e % 8) / 2] = __builtin_amdgcn_perm(__float_as_uint(l1), __float_as_uint(l0), 0x07060302u);
            }
        l_run = fmaf(l_run, alpha, psum);
        // the running maxima stop moving after the first tiles: skip the rescale when no row of the wave needs it
        if (__ballot(alpha != 1.0f) != 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[nb][e] *= alpha;
        }
        // O^T += V^T P^T
#pragma unroll
        for (int g16 = 0; g16 < 4; ++g16)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                BF8 va;
                const uint16_t *vrow = &sm.vt[buf][32 * nb + n][16 * g16 + 4 * h];
                const uint2 x0 = *reinterpret_cast<const uint2 *>(vrow), x1 = *reinterpret_cast<const uint2 *>(vrow + 8);
                va.u[0] = x0.x; va.u[1] = x0.y; va.u[2] = x1.x; va.u[3] = x1.y;
                oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.b, ph[g16].b, oacc[nb], 0, 0, 0);
                oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.b, pl[g16].b, oacc[nb], 0, 0, 0);
            }
        // stage the next tile into the other buffer, request the one after
        if (!stage_first && tile + 1 < tile_end) {
            stage_tile(buf ^ 1);
            load_tile(min(tile + 2, tile_end - 1));
        }
        __syncthreads();
    }

    // partial of each row: element e of block nb is channel 32 nb + 8 (e / 4) + 4 h + e % 4 of row n
    const int row = wave * 32 + n;
    const int grp = static_cast<int>(group_id % shp.n_row_groups);
    if (grp * ROWS + row < shp.rows_per_kv) {
        const int64_t prow = (group_id * ROWS + row) * shp.n_splits + split;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<float4 *>(part_acc + prow * D + 32 * nb + 8 * q4 + 4 * h) =
                    make_float4(oacc[nb][4 * q4], oacc[nb][4 * q4 + 1], oacc[nb][4 * q4 + 2], oacc[nb][4 * q4 + 3]);
        const float l = l_run + __shfl_xor(l_run, 32, kWave);
        if (h == 0) {
            part_ml[prow * 2] = m_run;
            part_ml[prow * 2 + 1] = l;
        }
    }
}

template <class P>
int launch_decode_mq(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                     const void *v, const int32_t *seq_lens, float *part_ml, float *part_acc, hipStream_t stream,
                     PageTable pt) {
    const DeviceBooks books = device_books(cb);
    const int64_t units = static_cast<int64_t>(s.n_seq) * s.n_kv_heads * s.n_splits;
    const int64_t wgs = (units + kXcds - 1) / kXcds * kXcds * s.n_row_groups;   // see the kernel's work mapping
    auto go = [&](auto kernel, int waves) {
        hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(wgs)), dim3(kWave * waves), 0, stream, books, s, q_rot,
                           static_cast<const uint4 *>(cache), static_cast<const uint16_t *>(v), seq_lens, part_ml, part_acc,
                           pt);
    };
    if (s.rows_per_pass == 128) {
        go(decode_kernel_mq<P, 4>, 4);
    } else if (s.rows_per_pass == 256) {
        if constexpr (P::D <= 64) go(decode_kernel_mq<P, 8>, 8);
        else return static_cast<int>(hipErrorInvalidValue);
    } else {
        return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

}  // namespace octopus

#endif
