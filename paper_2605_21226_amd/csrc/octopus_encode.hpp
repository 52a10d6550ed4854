// Online key encoder (Alg. 1 with the local 3x3 candidate set), one workgroup of 4 wavefronts per
// 64-token cache tile of one (sequence, KV head).
#ifndef OCTOPUS_ENCODE_HPP_
#define OCTOPUS_ENCODE_HPP_

#include "octopus_device.hpp"

namespace octopus {

constexpr int kURow = 65;  // words per coordinate row of the rotated tile (64 keys + 1 pad)

template <int D>
constexpr float inv_sqrt_dim() {
    return D == 64 ? 0.125f : (D == 128 ? 0.08838834764831845f : 0.0625f);
}

// Seed search (Alg. 1, searchsorted on B_xi) through a uniform grid of cells over [-1, 1]: a cell
// stores how many boundaries lie in lower cells and the first boundary not below the cell.  The host
// checks that no cell holds more than two boundaries, so two compares finish the count exactly.
template <int BD>
struct SeedGrid {
    static constexpr int K = 1 << BD;
    static constexpr int NCELL = 8 * K;
    __device__ static __forceinline__ int cell_of(float x) {
        const int c = static_cast<int>(floorf((x + 1.0f) * (0.5f * NCELL)));
        return min(max(c, 0), NCELL - 1);
    }
};

template <class P>
struct EncodeSmem {
    float u[3 * P::NTRI][kURow];           // rotated coordinates [coordinate][key]
    uint32_t rec[P::NWORDS][kWave];        // packed records [word][key]
    float4 lut0[P::LUT0];
    float4 lut1[P::LUT1 > 0 ? P::LUT1 : 1];
    float2 cell0[SeedGrid<P::BD0>::NCELL];
    float2 cell1[P::NCLASS == 2 ? SeedGrid<(P::BD1 > 0 ? P::BD1 : 1)>::NCELL : 1];
    float c_xi[2][32];
    float c_rho[2][8];
    float bnd_xi[2][33];                   // boundaries, +inf padded
    float bnd_rho[2][8];
    float inv_norm[kWave];
};

template <int BD>
__device__ __forceinline__ void build_seed_grid(float2 *cell, float *bnd, const float *c_xi, int tid, int nthreads) {
    using G = SeedGrid<BD>;
    for (int k = tid; k < 33; k += nthreads)
        bnd[k] = (k < G::K - 1) ? 0.5f * (c_xi[k] + c_xi[k + 1]) : INFINITY;
    for (int c = tid; c < G::NCELL; c += nthreads) {
        int below = 0;
        for (int k = 0; k < G::K - 1; ++k) {
            const float b = 0.5f * (c_xi[k] + c_xi[k + 1]);
            below += (G::cell_of(b) < c) ? 1 : 0;
        }
        const float first = (below < G::K - 1) ? 0.5f * (c_xi[below] + c_xi[below + 1]) : INFINITY;
        cell[c] = make_float2(__int_as_float(below), first);
    }
}

// number of boundaries strictly below x
template <int BD>
__device__ __forceinline__ int seed_index(const float2 *cell, const float *bnd, float x) {
    const float2 e = cell[SeedGrid<BD>::cell_of(x)];
    const int j = __float_as_int(e.x);
    return j + (e.y < x ? 1 : 0) + (bnd[j + 1] < x ? 1 : 0);
}

template <int R>
__device__ __forceinline__ void butterflies(float (&x)[R]) {
#pragma unroll
    for (int h = 1; h < R; h <<= 1) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if ((j & h) == 0) {
                const float a = x[j], b = x[j | h];
                x[j] = a + b;
                x[j | h] = a - b;
            }
        }
    }
}

// One triplet of one key: E4-E7 of the hot path.  Returns the packed direction field and norm index.
template <int BD, int BN>
__device__ __forceinline__ void encode_triplet(float x, float y, float z, const float4 *lut, const float2 *cell,
                                               const float *bnd_xi, const float *bnd_rho, uint32_t *dir_field,
                                               uint32_t *nrm_index) {
    constexpr int K = 1 << BD, M = 1 << BN;
    // Eq. (oct-encode)
    const float l1 = fabsf(x) + fabsf(y) + fabsf(z);
    const float inv = __builtin_amdgcn_rcpf(fmaxf(l1, kEps));
    const float px = x * inv, py = y * inv;
    float xi = px, eta = py;
    if (z < 0.0f) {
        const float fx = 1.0f - fabsf(py), fy = 1.0f - fabsf(px);
        xi = (px >= 0.0f) ? fx : -fx;
        eta = (py >= 0.0f) ? fy : -fy;
    }
    // scalar seed
    const int jx = seed_index<BD>(cell, bnd_xi, xi);
    const int jy = seed_index<BD>(cell, bnd_xi, eta);
    // local 3x3 joint rounding: dx outer, dy inner, strict '>' keeps the first maximum
    int ax[3] = {max(jx - 1, 0), jx, min(jx + 1, K - 1)};
    int ay[3] = {max(jy - 1, 0) << BD, jy << BD, min(jy + 1, K - 1) << BD};
    float best = -INFINITY;
    uint32_t best_code = 0;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const uint32_t code = static_cast<uint32_t>(ax[a] | ay[b]);
            const float4 n = lut[code];
            const float s = fmaf(z, n.z, fmaf(y, n.y, x * n.x));
            if (s > best) { best = s; best_code = code; }
        }
    }
    const float cs = fminf(fmaxf(best, 0.0f), 1.0f);
    int r = 0;
#pragma unroll
    for (int k = 0; k < M - 1; ++k) r += (bnd_rho[k] < cs) ? 1 : 0;
    *dir_field = best_code;
    *nrm_index = static_cast<uint32_t>(r);
}

__device__ __forceinline__ void or_bits(uint32_t (*rec)[kWave], int key, int bitpos, int nbits, uint32_t v) {
    const int wi = bitpos >> 5, sh = bitpos & 31;
    atomicOr(&rec[wi][key], v << sh);
    if (sh + nbits > 32) atomicOr(&rec[wi + 1][key], v >> (32 - sh));
}

template <class P, bool BF16>
__global__ __launch_bounds__(256) void encode_kernel(DeviceBooks books, const void *__restrict__ keys,
                                                      int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                                                      int32_t n_new, const uint8_t *__restrict__ signs,
                                                      uint4 *__restrict__ cache, int64_t t_capacity,
                                                      const int32_t *__restrict__ start_pos, int32_t n_kv_heads) {
    constexpr int D = P::D;
    constexpr int LPR = D / 8;        // threads per key row in the load phase
    constexpr int RPP = 256 / LPR;    // key rows per load pass
    extern __shared__ __align__(16) unsigned char smem_raw[];
    EncodeSmem<P> &sm = *reinterpret_cast<EncodeSmem<P> *>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kvh = blockIdx.y, seq = blockIdx.z;
    const int64_t start = start_pos ? start_pos[seq] : 0;
    const int64_t tile = start / kWave + blockIdx.x;
    const int64_t tok_lo = max(tile * kWave, start);
    const int64_t tok_hi = min(min((tile + 1) * kWave, start + n_new), t_capacity);
    if (tok_lo >= tok_hi) return;

    if (wave == 0) copy_books(books, sm.c_xi, sm.c_rho);
    for (int e = tid; e < P::NWORDS * kWave; e += 256) sm.rec[e / kWave][e % kWave] = 0u;
    for (int e = tid; e < (3 * P::NTRI - D) * kWave; e += 256) sm.u[D + e / kWave][e % kWave] = 0.0f;
    __syncthreads();

    // tables
    build_dir_lut<P::BD0>(sm.lut0, sm.c_xi[0], tid, 256);
    build_seed_grid<P::BD0>(sm.cell0, sm.bnd_xi[0], sm.c_xi[0], tid, 256);
    if constexpr (P::NCLASS == 2) {
        build_dir_lut<P::BD1>(sm.lut1, sm.c_xi[1], tid, 256);
        build_seed_grid<P::BD1>(sm.cell1, sm.bnd_xi[1], sm.c_xi[1], tid, 256);
    }
    if (tid < 16) {
        const int c = tid >> 3, k = tid & 7;
        sm.bnd_rho[c][k] = (k < 7) ? 0.5f * (sm.c_rho[c][k] + sm.c_rho[c][k + 1]) : INFINITY;
    }

    // E1-E2: load, squared norm, sign flip
    const int64_t head_base = seq * stride_seq + kvh * stride_head;
    const int col = (tid % LPR) * 8;
    const uint32_t sbits = signs[kvh * (D / 8) + col / 8];
#pragma unroll
    for (int pass = 0; pass < kWave / RPP; ++pass) {
        const int key = pass * RPP + tid / LPR;
        const int64_t tok = tile * kWave + key;
        const bool valid = tok >= tok_lo && tok < tok_hi;
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.0f;
        if (valid) {
            const int64_t off = head_base + (tok - start) * stride_tok + col;
            if constexpr (BF16) {
                const uint4 r = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(keys) + off);
                x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
                x[4] = bf16_lo(r.z); x[5] = bf16_hi(r.z); x[6] = bf16_lo(r.w); x[7] = bf16_hi(r.w);
            } else {
                const float4 a = *reinterpret_cast<const float4 *>(static_cast<const float *>(keys) + off);
                const float4 b = *reinterpret_cast<const float4 *>(static_cast<const float *>(keys) + off + 4);
                x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
            }
        }
        float ss = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o, kWave);
#pragma unroll
        for (int e = 0; e < 8; ++e) sm.u[col + e][key] = ((sbits >> e) & 1u) ? -x[e] : x[e];
        if (tid % LPR == 0) {
            const float gamma = sqrtf(ss);
            sm.rec[0][key] = __float_as_uint(gamma);
            sm.inv_norm[key] = (1.0f / fmaxf(gamma, kEps)) * inv_sqrt_dim<D>();
        }
    }
    __syncthreads();

    // E3: Walsh-Hadamard transform, one key per lane, two radix passes through LDS
    {
        constexpr int R2 = D / 16;
        for (int g = wave; g < D / 16; g += 4) {
            float x[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) x[e] = sm.u[g * 16 + e][lane];
            butterflies<16>(x);
#pragma unroll
            for (int e = 0; e < 16; ++e) sm.u[g * 16 + e][lane] = x[e];
        }
        __syncthreads();
        const float norm = sm.inv_norm[lane];
        for (int lo = wave; lo < 16; lo += 4) {
            float x[R2];
#pragma unroll
            for (int e = 0; e < R2; ++e) x[e] = sm.u[e * 16 + lo][lane];
            butterflies<R2>(x);
#pragma unroll
            for (int e = 0; e < R2; ++e) sm.u[e * 16 + lo][lane] = x[e] * norm;
        }
        __syncthreads();
    }

    // E4-E8: triplets, a quarter of them per wavefront, one key per lane
    {
        constexpr int CHUNK = (P::NTRI + 3) / 4;
        const int i_end = min(P::NTRI, (wave + 1) * CHUNK);
        for (int i = wave * CHUNK; i < i_end; ++i) {
            const float x = sm.u[3 * i][lane], y = sm.u[3 * i + 1][lane], z = sm.u[3 * i + 2][lane];
            uint32_t dir_field, nrm_index;
            if (P::NCLASS == 1 || i < P::NT0) {
                encode_triplet<P::BD0, P::BN0>(x, y, z, sm.lut0, sm.cell0, sm.bnd_xi[0], sm.bnd_rho[0], &dir_field,
                                               &nrm_index);
                or_bits(sm.rec, lane, P::DIR0_BIT + i * 2 * P::BD0, 2 * P::BD0, dir_field);
                or_bits(sm.rec, lane, P::NRM0_BIT + i * P::BN0, P::BN0, nrm_index);
            } else {
                if constexpr (P::NCLASS == 2) {
                    encode_triplet<P::BD1, P::BN1>(x, y, z, sm.lut1, sm.cell1, sm.bnd_xi[1], sm.bnd_rho[1],
                                                   &dir_field, &nrm_index);
                    or_bits(sm.rec, lane, P::DIR1_BIT + (i - P::NT0) * 2 * P::BD1, 2 * P::BD1, dir_field);
                    or_bits(sm.rec, lane, P::NRM1_BIT + (i - P::NT0) * P::BN1, P::BN1, nrm_index);
                }
            }
        }
    }
    __syncthreads();

    // E8: store the tile, 16 bytes per (granule, key), coalesced over keys
    uint4 *region = cache + (static_cast<int64_t>(seq) * n_kv_heads + kvh) * (t_capacity * P::GRANULES) +
                    tile * (P::GRANULES * kWave);
    for (int e = tid; e < P::GRANULES * kWave; e += 256) {
        const int g = e / kWave, key = e % kWave;
        const int64_t tok = tile * kWave + key;
        if (tok >= tok_lo && tok < tok_hi)
            region[e] = make_uint4(sm.rec[4 * g][key], sm.rec[4 * g + 1][key], sm.rec[4 * g + 2][key],
                                   sm.rec[4 * g + 3][key]);
    }
}

template <class P>
int launch_encode_plan(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                       int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                       const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                       hipStream_t stream) {
    DeviceBooks books;
    for (int c = 0; c < 2; ++c) {
        for (int k = 0; k < 32; ++k) books.c_xi[c][k] = cb.c_xi[c][k];
        for (int k = 0; k < 8; ++k) books.c_rho[c][k] = cb.c_rho[c][k];
    }
    // a start that is not a multiple of 64 makes the new tokens straddle one more tile
    const int tiles = (n_new + kWave - 1) / kWave + (start_pos ? 1 : 0);
    const dim3 grid(tiles, n_kv_heads, n_seq);
    const size_t smem = sizeof(EncodeSmem<P>);
    hipError_t err;
    if (key_dtype == OCTOPUS_DTYPE_BF16) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&encode_kernel<P, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
        if (err != hipSuccess) return static_cast<int>(err);
        hipLaunchKernelGGL((encode_kernel<P, true>), grid, dim3(256), smem, stream, books, keys, stride_seq,
                           stride_tok, stride_head, n_new, signs, static_cast<uint4 *>(cache), t_capacity, start_pos,
                           n_kv_heads);
    } else {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&encode_kernel<P, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
        if (err != hipSuccess) return static_cast<int>(err);
        hipLaunchKernelGGL((encode_kernel<P, false>), grid, dim3(256), smem, stream, books, keys, stride_seq,
                           stride_tok, stride_head, n_new, signs, static_cast<uint4 *>(cache), t_capacity, start_pos,
                           n_kv_heads);
    }
    return static_cast<int>(hipGetLastError());
}

}  // namespace octopus

#endif
