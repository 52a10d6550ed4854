// Online key encoder (Alg. 1 with the local 3x3 candidate set): a workgroup of 4 or 8 wavefronts takes one to
// eight consecutive 64-token cache tiles of one (sequence, KV head), one after the other.
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
// stores how many boundaries lie in lower cells and the boundary inside the cell (+inf if none).  The
// host refuses codebooks with two boundaries in one cell, so one compare finishes the count exactly:
// the cell index is monotone in x, hence boundaries of lower cells are below x and those of higher
// cells above it.
template <int BD>
struct SeedGrid {
    static constexpr int K = 1 << BD;
    static constexpr int NCELL = 8 * K;
    __device__ static __forceinline__ int cell_of(float x) {
        // floor((x + 1) * NCELL / 2), clamped: the scaling by a power of two is exact, so one fused multiply-add
        // rounds as the sum does, and the conversion's truncation is the floor wherever the clamp lets it through
        const int c = static_cast<int>(fmaf(x, 0.5f * NCELL, 0.5f * NCELL));
        return min(max(c, 0), NCELL - 1);
    }
};

// The direction table holds ONE QUADRANT of the code grid: a Lloyd-Max codebook of the symmetric marginal is
// antisymmetric (C_xi[K - 1 - j] = -C_xi[j], checked on the host), and Oct^-1(-xi, eta) is Oct^-1(xi, eta) with
// its first component negated, bit for bit (likewise eta and the second component).  Entry (fx, fy), fx, fy <
// K / 2, is Oct^-1(C_xi[fx], C_xi[fy]); a code (jx, jy) reads entry (min(jx, K-1-jx), min(jy, K-1-jy)) and negates
// the key's x (y) coordinate instead of the entry's when jx (jy) lies in the upper half -- the products, and so
// the scores, are the same numbers.  A quarter of the entries pays for four times the copies: copy r of entry
// e sits at index e * REP + r and lane l reads copy l % REP, so with 8 copies of 16 bytes any 8 neighbouring lanes
// read 8 different groups of banks whatever their codes (two copies of the full table left the candidate reads
// with about one conflict cycle per useful cycle).  For 6-bit direction codes four copies fit the budget; at
// d = 256, where the rotated tile alone takes 67 KB, four copies up to 3-bit codes and two above, so that two
// workgroups still fit a compute unit at 3 bits per coordinate.  The seed grid keeps two copies up to d = 128.
template <int D, int BD = 1>
constexpr int encode_table_rep() { return (D <= 128 && BD <= 5) ? 8 : (D <= 128 || BD <= 3 ? 4 : 2); }
template <int D>
constexpr int encode_cell_rep() { return D <= 128 ? 2 : 1; }
constexpr int quadrant_entries(int bd) { return bd <= 1 ? 1 : (1 << (2 * (bd - 1))); }

// Wavefronts per workgroup.  LDS (the rotated tile, above all) decides how many workgroups a compute unit holds:
// three at d = 128 up to 3 bits per coordinate, two at 4 bits and at d = 256, one at d = 256 and 4 bits; with four
// wavefronts each a SIMD then has three, two or one to choose from, and the kernel waits on LDS and barriers.  Eight
// wavefronts share a tile from d = 128 on (measured, same records: d = 128 b = 3 -4 %, b = 4 -15 %; d = 256 b = 3
// -8 %, b = 4 -28 %; at d = 64 four workgroups fit anyway and eight wavefronts gain nothing).
template <class P>
constexpr int encode_waves() { return P::D >= 128 ? 8 : 4; }
template <class P>
constexpr int encode_threads() { return encode_waves<P>() * kWave; }

template <class P, bool QJL = false>
struct EncodeSmem {
    float u[3 * P::NTRI][kURow];           // rotated coordinates [coordinate][key]
    uint32_t rec[P::NWORDS][kWave];        // packed records [word][key]
    static constexpr int REP = encode_table_rep<P::D, (P::BD0 > P::BD1 ? P::BD0 : P::BD1)>();
    static constexpr int CREP = encode_cell_rep<P::D>();
    float4 lut0[quadrant_entries(P::BD0) * REP];
    float4 lut1[P::NCLASS == 2 ? quadrant_entries(P::BD1) * REP : 1];
    float2 cell0[SeedGrid<P::BD0>::NCELL * CREP];
    float2 cell1[P::NCLASS == 2 ? SeedGrid<(P::BD1 > 0 ? P::BD1 : 1)>::NCELL * CREP : 1];
    // neighbours of a seed index j on the x and on the y axis, [j][dx + 1]: {+-1 (the sign the key's coordinate
    // takes), byte offset of the candidate's row / column in the quadrant table}
    float2 nbx0[(1 << P::BD0) * 3], nby0[(1 << P::BD0) * 3];
    float2 nbx1[P::NCLASS == 2 ? (1 << P::BD1) * 3 : 1], nby1[P::NCLASS == 2 ? (1 << P::BD1) * 3 : 1];
    float c_xi[2][kMaxLevels];
    float c_rho[2][kMaxLevels];
    float bnd_xi[2][kMaxLevels + 1];       // boundaries, +inf padded
    float bnd_rho[2][kMaxLevels];
    float sumsq[kWave];                    // squared norm of each key of the tile, then its scale factor 1 / (gamma sqrt(d))
    float res_sq[QJL ? encode_waves<P>() : 1][QJL ? kWave : 1];   // QJL side-car: squared residual norm, partial per wavefront
};

// Wavefronts per SIMD that the LDS footprint allows (160 KB per compute unit, 4 SIMDs): the register budget the
// kernel is compiled for, so that registers never cost a workgroup that LDS has room for.
template <class P, bool QJL>
constexpr int encode_waves_per_simd() {
    constexpr int groups = static_cast<int>((160 * 1024) / sizeof(EncodeSmem<P, QJL>));
    constexpr int waves = (groups < 1 ? 1 : groups) * encode_waves<P>() / 4;
    return waves > 6 ? 6 : waves;   // (the kernel does not fit the 64 registers of 8 wavefronts per SIMD)
}

template <int BD, int REP>
__device__ __forceinline__ void build_encode_lut(float4 *lut, float2 *nbx, float2 *nby, const float *c_xi, int tid,
                                                 int nthreads) {
    constexpr int K = 1 << BD, H = BD <= 1 ? 1 : K / 2;
    // (with fewer entries than threads, nthreads / (H * H) threads share an entry: each computes it once and
    // writes its share of the copies)
    constexpr int Q = H * H;
    if (Q >= nthreads) {
        for (int e = tid; e < Q; e += nthreads) {
            const float4 n = oct_decode(c_xi[e % H], c_xi[e / H]);
#pragma unroll
            for (int r = 0; r < REP; ++r) lut[e * REP + r] = n;
        }
    } else {
        const int per_entry = nthreads / Q, e = tid % Q;
        const float4 n = oct_decode(c_xi[e % H], c_xi[e / H]);
        for (int r = tid / Q; r < REP; r += per_entry) lut[e * REP + r] = n;
    }
    for (int e = tid; e < 3 * K; e += nthreads) {
        const int j = min(max(e / 3 + e % 3 - 1, 0), K - 1);   // the clamped neighbour (Alg. 1's window at the rim)
        const int f = min(j, K - 1 - j);
        const float sign = j >= H && K > 1 ? -1.0f : 1.0f;
        nbx[e] = make_float2(sign, __uint_as_float(static_cast<uint32_t>(f * REP * 16)));
        nby[e] = make_float2(sign, __uint_as_float(static_cast<uint32_t>(f * H * REP * 16)));
    }
}

// Oct^-1 of the centroids of a direction code, from the quadrant table.
template <int BD, int REP>
__device__ __forceinline__ float4 dir_lookup(const float4 *lut, uint32_t code, int lane) {
    constexpr int K = 1 << BD, H = BD <= 1 ? 1 : K / 2;
    const int jx = static_cast<int>(code & (K - 1)), jy = static_cast<int>(code >> BD);
    const int fx = min(jx, K - 1 - jx), fy = min(jy, K - 1 - jy);
    float4 n = lut[(fx + fy * H) * REP + (lane & (REP - 1))];
    if (jx >= H) n.x = -n.x;
    if (jy >= H) n.y = -n.y;
    return n;
}

template <int BD, int REP>
__device__ __forceinline__ void build_seed_grid(float2 *cell, float *bnd, const float *c_xi, int tid, int nthreads) {
    using G = SeedGrid<BD>;
    for (int k = tid; k <= kMaxLevels; k += nthreads)
        bnd[k] = (k < G::K - 1) ? 0.5f * (c_xi[k] + c_xi[k + 1]) : INFINITY;
    for (int c = tid; c < G::NCELL; c += nthreads) {
        int below = 0;
        for (int k = 0; k < G::K - 1; ++k) {
            const float b = 0.5f * (c_xi[k] + c_xi[k + 1]);
            below += (G::cell_of(b) < c) ? 1 : 0;
        }
        const float first = (below < G::K - 1) ? 0.5f * (c_xi[below] + c_xi[below + 1]) : INFINITY;
#pragma unroll
        for (int r = 0; r < REP; ++r) cell[c * REP + r] = make_float2(__int_as_float(below), first);
    }
}

// number of boundaries strictly below x
template <int BD, int REP>
__device__ __forceinline__ int seed_index(const float2 *cell, const float *bnd, float x, int lane) {
    (void)bnd;
    const float2 e = cell[SeedGrid<BD>::cell_of(x) * REP + (lane & (REP - 1))];
    return __float_as_int(e.x) + (e.y < x ? 1 : 0);
}

// Sum over the LPR (8, 16 or 32) neighbouring lanes that hold one key row, left in all of them: an exchange-and-add
// butterfly over lane distances 1, 2, 4, 8 (and 16).  The first four go through the vector ALU's own lane permutes
// instead of LDS: after the distances 1 and 2 the four lanes of a quad hold the same sum, so the mirror of 8 lanes
// pairs each quad with its neighbour exactly as distance 4 does, and the mirror of 16 each half as distance 8 does
// (the same two operands in every addition, so the same bits).
template <int CTRL>
__device__ __forceinline__ float lane_permute(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
    static_assert(LPR == 8 || LPR == 16 || LPR == 32, "lanes per key row");
    v += lane_permute<0xB1>(v);    // quad permute [1, 0, 3, 2]
    v += lane_permute<0x4E>(v);    // quad permute [2, 3, 0, 1]
    v += lane_permute<0x141>(v);   // mirror within each 8 lanes
    if constexpr (LPR >= 16) v += lane_permute<0x140>(v);   // mirror within each 16 lanes
    if constexpr (LPR >= 32) v += __shfl_xor(v, 16, kWave);
    return v;
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
template <int BD, int BN, int REP, int CREP>
__device__ __forceinline__ void encode_triplet(float x, float y, float z, const float4 *lut, const float2 *cell,
                                               const float2 *nbx, const float2 *nby, const float *bnd_xi,
                                               const float *bnd_rho, int lane, uint32_t *dir_field,
                                               uint32_t *nrm_index) {
    constexpr int K = 1 << BD, M = 1 << BN;
    // Eq. (oct-encode)
    const float l1 = fabsf(x) + fabsf(y) + fabsf(z);
    // 1 / l1: the hardware reciprocal (1 ulp) refined by one Newton step, so that xi and eta carry the rounding of
    // a division rather than of an approximation (they are compared with the codebook boundaries below)
    const float l1c = fmaxf(l1, kEps);
    float inv = __builtin_amdgcn_rcpf(l1c);
    inv = fmaf(fmaf(-l1c, inv, 1.0f), inv, inv);
    const float px = x * inv, py = y * inv;
    float xi = px, eta = py;
    if (z < 0.0f) {
        const float fx = 1.0f - fabsf(py), fy = 1.0f - fabsf(px);
        xi = (px >= 0.0f) ? fx : -fx;
        eta = (py >= 0.0f) ? fy : -fy;
    }
    // scalar seed
    const int jx = seed_index<BD, CREP>(cell, bnd_xi, xi, lane);
    const int jy = seed_index<BD, CREP>(cell, bnd_xi, eta, lane);
    // local 3x3 joint rounding: dx outer, dy inner, the first maximum wins
    // the candidates' places in the quadrant table and the signs the key's coordinates take for them
    // (24-bit multiplies: full rate, unlike the 32-bit one)
    const float2 *rowx = reinterpret_cast<const float2 *>(reinterpret_cast<const char *>(nbx) + __mul24(jx, 24));
    const float2 *rowy = reinterpret_cast<const float2 *>(reinterpret_cast<const char *>(nby) + __mul24(jy, 24));
    float xa[3], yb[3];
    uint32_t ox[3], oy[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const float2 ex = rowx[a], ey = rowy[a];
        xa[a] = x * ex.x;
        ox[a] = __float_as_uint(ex.y);
        yb[a] = y * ey.x;
        oy[a] = __float_as_uint(ey.y);
    }
    const char *base = reinterpret_cast<const char *>(lut) + (lane & (REP - 1)) * 16;
    // all nine scores, their maximum, then the first candidate that attains it
    float sc[9];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const float4 n = *reinterpret_cast<const float4 *>(base + ox[a] + oy[b]);
            sc[3 * a + b] = fmaf(z, n.z, fmaf(yb[b], n.y, xa[a] * n.x));
        }
    }
    // the maximum per dx, then overall; the winner is the first dx whose maximum attains it and, of that dx's three
    // candidates, the first that does (the order of Alg. 1's loop: dx outer, dy inner), found with two compares per
    // level instead of one per candidate
    const float row0 = fmaxf(fmaxf(sc[0], sc[1]), sc[2]), row1 = fmaxf(fmaxf(sc[3], sc[4]), sc[5]),
                row2 = fmaxf(fmaxf(sc[6], sc[7]), sc[8]);
    const float best = fmaxf(fmaxf(row0, row1), row2);
    const bool in0 = row0 == best, in1 = row1 == best;
    const int pick_x = in0 ? 0 : (in1 ? 1 : 2);
    const float first = in0 ? sc[0] : (in1 ? sc[3] : sc[6]), second = in0 ? sc[1] : (in1 ? sc[4] : sc[7]);
    const int pick_y = first == best ? 0 : (second == best ? 1 : 2);
    const int cx = min(max(jx + pick_x - 1, 0), K - 1);
    const int cy = min(max(jy + pick_y - 1, 0), K - 1);
    const uint32_t best_code = static_cast<uint32_t>(cx | (cy << BD));
    const float cs = fminf(fmaxf(best, 0.0f), 1.0f);
    int r = 0;
#pragma unroll
    for (int k = 0; k < M - 1; ++k) r += (bnd_rho[k] < cs) ? 1 : 0;
    *dir_field = best_code;
    *nrm_index = static_cast<uint32_t>(r);
}

// The encoder-only rounding variants of App. E (same bitstream, same decoder); `mode` as in octopus.h:
// 0 seed only (Alg. 1 with the window {(0,0)}), 1 local 3x3, 2 full K x K grid, 3 three independent
// nearest-centroid rounds (the norm code from rho_i itself), 4 local 2x2 (the seed and its upper neighbour).
// Candidates are visited dx outer, dy inner (full grid: x index outer); the first maximum wins.
template <int BD, int BN, int REP, int CREP>
__device__ __forceinline__ void encode_triplet_any(float x, float y, float z, const float4 *lut, const float2 *cell,
                                                   const float *bnd_xi, const float *bnd_rho, int lane, int mode,
                                                   uint32_t *dir_field, uint32_t *nrm_index) {
    constexpr int K = 1 << BD, M = 1 << BN;
    const float l1 = fabsf(x) + fabsf(y) + fabsf(z);
    // 1 / l1: the hardware reciprocal (1 ulp) refined by one Newton step, so that xi and eta carry the rounding of
    // a division rather than of an approximation (they are compared with the codebook boundaries below)
    const float l1c = fmaxf(l1, kEps);
    float inv = __builtin_amdgcn_rcpf(l1c);
    inv = fmaf(fmaf(-l1c, inv, 1.0f), inv, inv);
    const float px = x * inv, py = y * inv;
    float xi = px, eta = py;
    if (z < 0.0f) {
        const float fx = 1.0f - fabsf(py), fy = 1.0f - fabsf(px);
        xi = (px >= 0.0f) ? fx : -fx;
        eta = (py >= 0.0f) ? fy : -fy;
    }
    const int jx = seed_index<BD, CREP>(cell, bnd_xi, xi, lane);
    const int jy = seed_index<BD, CREP>(cell, bnd_xi, eta, lane);
    float best = -INFINITY;
    uint32_t best_code = 0u;
    auto consider = [&](int ax, int ay) {
        const uint32_t code = static_cast<uint32_t>(ax | (ay << BD));
        const float4 n = dir_lookup<BD, REP>(lut, code, lane);
        const float sc = fmaf(z, n.z, fmaf(y, n.y, x * n.x));
        if (sc > best) { best = sc; best_code = code; }
    };
    // rolled loops on purpose: these variants are for ablations, and unrolling K x K candidates per
    // triplet of every class blows the code up
    if (mode == 2) {
#pragma clang loop unroll(disable)
        for (int c = 0; c < K * K; ++c) consider(c >> BD, c & (K - 1));
    } else {
        const int lo = (mode == 1) ? -1 : 0;
        const int hi = (mode == 1 || mode == 4) ? 1 : 0;
#pragma clang loop unroll(disable)
        for (int dx = lo; dx <= hi; ++dx)
#pragma clang loop unroll(disable)
            for (int dy = lo; dy <= hi; ++dy) consider(min(max(jx + dx, 0), K - 1), min(max(jy + dy, 0), K - 1));
    }
    const float radial = (mode == 3) ? sqrtf(fmaf(z, z, fmaf(y, y, x * x))) : best;
    const float cs = fminf(fmaxf(radial, 0.0f), 1.0f);
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

// Consecutive cache tiles one workgroup takes, its tables built once for all of them: eight where that still leaves
// the launch several workgroups per place on the chip (a long prefill: the tables cost a fifth of a tile's time),
// fewer for shorter calls, down to one, so that a short chunk still spreads over the compute units.
inline int encode_tiles_per_group(int tiles, int n_kv_heads, int n_seq) {
    constexpr int64_t kEnough = 3072;   // 256 compute units x 3 resident workgroups x 4
    for (int t = 8; t > 1; t >>= 1)
        if (static_cast<int64_t>((tiles + t - 1) / t) * n_kv_heads * n_seq >= kEnough) return t;
    return 1;
}

// QJL: also write the optional side-car of Sec. 3.6 (1-bit QJL residual): the residual r = u - u^ of the
// rotated unit key replaces u in LDS as the triplets are encoded, a second sign-flipped Hadamard
// transform follows, and the signs of its output (bit set = negative) plus ||r|| as fp16 are stored per
// key: per tile of 64 tokens [d/32 words][64 keys] uint32, then [64 keys] fp16.
// ANY: the rounding mode is the run-time argument `mode` (the default encoder is built without it).
template <class P, bool BF16, bool QJL, bool ANY = false>
__global__ __launch_bounds__(encode_threads<P>())
__attribute__((amdgpu_waves_per_eu(encode_waves_per_simd<P, QJL>(), encode_waves_per_simd<P, QJL>())))
void encode_kernel(DeviceBooks books, const void *__restrict__ keys,
                                                      int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                                                      int32_t n_new, const uint8_t *__restrict__ signs,
                                                      uint4 *__restrict__ cache, int64_t t_capacity,
                                                      const int32_t *__restrict__ start_pos, int32_t n_kv_heads,
                                                      const uint8_t *__restrict__ signs2,
                                                      unsigned char *__restrict__ qjl, int32_t mode, PageTable pt,
                                                      int32_t tiles_per_group) {
    constexpr int D = P::D;
    constexpr int LPR = D / 8;        // threads per key row in the load phase
    constexpr int NWV = encode_waves<P>(), NT = encode_threads<P>();
    constexpr int RPP = NT / LPR;     // key rows per load pass
    constexpr int REP = EncodeSmem<P, QJL>::REP, CREP = EncodeSmem<P, QJL>::CREP;
    // static, so that table addresses are compile-time constants that fold into the LDS instructions
    __shared__ EncodeSmem<P, QJL> sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int kvh = blockIdx.y, seq = blockIdx.z;
    const int64_t start = start_pos ? max(start_pos[seq], 0) : 0;   // (a negative position would write before the cache)
    const int64_t tok_end = min(start + n_new, t_capacity);
    const int64_t first_tile = start / kWave + static_cast<int64_t>(blockIdx.x) * tiles_per_group;
    if (max(first_tile * kWave, start) >= tok_end) return;

    const int64_t head_base = seq * stride_seq + kvh * stride_head;
    const int col = (tid % LPR) * 8;
    const uint32_t sbits = signs[kvh * (D / 8) + col / 8];
    uint4 *region = cache + (static_cast<int64_t>(seq) * n_kv_heads + kvh) * (t_capacity * P::GRANULES);

    // A tile's key rows as loaded: 8 coordinates per thread and pass (bf16: one 16-byte word; fp32: two);
    // rows outside [start, tok_end) and tiles past the group's last one read as zeros.  The next tile's rows
    // are requested as soon as the current ones sit in LDS, so that they arrive during its transform and
    // triplet phases.
    constexpr int NPASS = kWave / RPP;
    uint4 raw[NPASS][BF16 ? 1 : 2];
    auto fetch_tile = [&](int64_t tile) {
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            const int64_t tok = tile * kWave + pass * RPP + tid / LPR;
            const bool valid = tok >= start && tok < tok_end;
#pragma unroll
            for (int h = 0; h < (BF16 ? 1 : 2); ++h) raw[pass][h] = make_uint4(0u, 0u, 0u, 0u);
            if (valid) {
                const int64_t off = head_base + (tok - start) * stride_tok + col;
                if constexpr (BF16) {
                    // 16 threads read one whole 256- or 512-byte row: streamed, read once (non-temporal)
                    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                    const u32x4_t x = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4_t *>(static_cast<const uint16_t *>(keys) + off));
                    raw[pass][0] = make_uint4(x.x, x.y, x.z, x.w);
                } else {
                    raw[pass][0] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(keys) + off);
                    raw[pass][BF16 ? 0 : 1] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(keys) + off + 4);
                }
            }
        }
    };
    // the first tile's rows are requested before the tables are built, so that they arrive meanwhile
    fetch_tile(first_tile);

    // tables
    if (wave == 0) copy_books<P>(books, sm.c_xi, sm.c_rho);
    __syncthreads();
    build_encode_lut<P::BD0, REP>(sm.lut0, sm.nbx0, sm.nby0, sm.c_xi[0], tid, NT);
    build_seed_grid<P::BD0, CREP>(sm.cell0, sm.bnd_xi[0], sm.c_xi[0], tid, NT);
    if constexpr (P::NCLASS == 2) {
        build_encode_lut<P::BD1, REP>(sm.lut1, sm.nbx1, sm.nby1, sm.c_xi[1], tid, NT);
        build_seed_grid<P::BD1, CREP>(sm.cell1, sm.bnd_xi[1], sm.c_xi[1], tid, NT);
    }
    if (tid < 2 * kMaxLevels) {
        const int c = tid / kMaxLevels, k = tid % kMaxLevels;
        const int levels = 1 << (c ? (P::BN1 > 0 ? P::BN1 : 1) : P::BN0);
        sm.bnd_rho[c][k] = (k < levels - 1) ? 0.5f * (sm.c_rho[c][k] + sm.c_rho[c][k + 1]) : INFINITY;
    }
    for (int e = tid; e < (3 * P::NTRI - D) * kWave; e += NT) sm.u[D + e / kWave][e % kWave] = 0.0f;

    for (int tg = 0; tg < tiles_per_group; ++tg) {
        const int64_t tile = first_tile + tg;
        const int64_t tok_lo = max(tile * kWave, start);
        const int64_t tok_hi = min((tile + 1) * kWave, tok_end);
        if (tok_lo >= tok_hi) break;   // uniform over the workgroup
        // paged cache: the tile's page is asked for now and used when the tile is stored, phases later
        int page_asked = 0;
        if (pt.table != nullptr) page_asked = pt.table[static_cast<int64_t>(seq) * pt.stride + tile];
        __syncthreads();               // the previous tile's records have been stored; tables are complete
        // word 0 (gamma) is written whole by the transform phase below; the code words are OR-ed into
        for (int e = kWave + tid; e < P::NWORDS * kWave; e += NT) sm.rec[e / kWave][e % kWave] = 0u;

        // E1-E2: squared norm, sign flip
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            const int key = pass * RPP + tid / LPR;
            float x[8];
            if constexpr (BF16) {
                const uint4 r = raw[pass][0];
                x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
                x[4] = bf16_lo(r.z); x[5] = bf16_hi(r.z); x[6] = bf16_lo(r.w); x[7] = bf16_hi(r.w);
            } else {
                const uint4 a = raw[pass][0], b = raw[pass][BF16 ? 0 : 1];
                x[0] = __uint_as_float(a.x); x[1] = __uint_as_float(a.y); x[2] = __uint_as_float(a.z);
                x[3] = __uint_as_float(a.w); x[4] = __uint_as_float(b.x); x[5] = __uint_as_float(b.y);
                x[6] = __uint_as_float(b.z); x[7] = __uint_as_float(b.w);
            }
            float ss = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
            ss = row_sum<LPR>(ss);
#pragma unroll
            for (int e = 0; e < 8; ++e) sm.u[col + e][key] = ((sbits >> e) & 1u) ? -x[e] : x[e];
            if (tid % LPR == 0) sm.sumsq[key] = ss;
        }
        if (tg + 1 < tiles_per_group) fetch_tile(tile + 1);
        __syncthreads();

        // E3: Walsh-Hadamard transform, one key per lane, two radix passes through LDS
        {
            constexpr int R2 = D / 16;
            // the norm of every key, once per key: by one wavefront, 64 keys at a time (the load phase has 4 to 32
            // lanes per key, and a square root and a division cost as much there for one active lane as for 64); the
            // scale factor replaces the sum of squares in LDS and is read by all after the barrier between the passes
            if (wave == NWV - 1) {
                const float gamma = sqrtf(sm.sumsq[lane]);
                sm.rec[0][lane] = __float_as_uint(gamma);
                sm.sumsq[lane] = (1.0f / fmaxf(gamma, kEps)) * inv_sqrt_dim<D>();
            }
            for (int g = wave; g < D / 16; g += NWV) {
                float x[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) x[e] = sm.u[g * 16 + e][lane];
                butterflies<16>(x);
#pragma unroll
                for (int e = 0; e < 16; ++e) sm.u[g * 16 + e][lane] = x[e];
            }
            __syncthreads();
            const float norm = sm.sumsq[lane];
            for (int lo = wave; lo < 16; lo += NWV) {
                float x[R2];
#pragma unroll
                for (int e = 0; e < R2; ++e) x[e] = sm.u[e * 16 + lo][lane];
                butterflies<R2>(x);
#pragma unroll
                for (int e = 0; e < R2; ++e) sm.u[e * 16 + lo][lane] = x[e] * norm;
            }
            __syncthreads();
        }

        // E4-E8: triplets, an equal share of them per wavefront, one key per lane
        {
            constexpr int CHUNK = (P::NTRI + NWV - 1) / NWV;
            const int i_end = min(P::NTRI, (wave + 1) * CHUNK);
            float rsq = 0.0f;
            // The norm thresholds of the default encoder in registers where they are few (up to 3 norm bits; the loop's
            // LDS atomics keep the compiler from hoisting the read itself, and LDS is this kernel's limit); with more
            // levels they stay in LDS, as registers are what six wavefronts per SIMD have least of.
            constexpr bool THR0_REG = P::BN0 <= 3, THR1_REG = P::NCLASS == 2 && P::BN1 >= 1 && P::BN1 <= 3;
            float thr0_reg[THR0_REG ? (1 << P::BN0) : 1], thr1_reg[THR1_REG ? (1 << P::BN1) : 1];
            if constexpr (THR0_REG) {
#pragma unroll
                for (int k = 0; k < (1 << P::BN0) - 1; ++k) thr0_reg[k] = sm.bnd_rho[0][k];
            }
            if constexpr (THR1_REG) {
#pragma unroll
                for (int k = 0; k < (1 << P::BN1) - 1; ++k) thr1_reg[k] = sm.bnd_rho[1][k];
            }
            const float *thr0 = THR0_REG ? thr0_reg : sm.bnd_rho[0];
            const float *thr1 = THR1_REG ? thr1_reg : sm.bnd_rho[1];
            for (int i = wave * CHUNK; i < i_end; ++i) {
                const float x = sm.u[3 * i][lane], y = sm.u[3 * i + 1][lane], z = sm.u[3 * i + 2][lane];
                uint32_t dir_field, nrm_index;
                float4 nhat;
                float rho;
                if (P::NCLASS == 1 || i < P::NT0) {
                    if constexpr (ANY)
                        encode_triplet_any<P::BD0, P::BN0, REP, CREP>(x, y, z, sm.lut0, sm.cell0, sm.bnd_xi[0],
                                                                      sm.bnd_rho[0], lane, mode, &dir_field, &nrm_index);
                    else
                        encode_triplet<P::BD0, P::BN0, REP, CREP>(x, y, z, sm.lut0, sm.cell0, sm.nbx0, sm.nby0,
                                                                  sm.bnd_xi[0], thr0, lane, &dir_field, &nrm_index);
                    or_bits(sm.rec, lane, P::DIR0_BIT + i * 2 * P::BD0, 2 * P::BD0, dir_field);
                    or_bits(sm.rec, lane, P::NRM0_BIT + i * P::BN0, P::BN0, nrm_index);
                    if constexpr (QJL) { nhat = dir_lookup<P::BD0, REP>(sm.lut0, dir_field, lane); rho = sm.c_rho[0][nrm_index]; }
                } else {
                    if constexpr (P::NCLASS == 2) {
                        if constexpr (ANY)
                            encode_triplet_any<P::BD1, P::BN1, REP, CREP>(x, y, z, sm.lut1, sm.cell1, sm.bnd_xi[1],
                                                                          sm.bnd_rho[1], lane, mode, &dir_field, &nrm_index);
                        else
                            encode_triplet<P::BD1, P::BN1, REP, CREP>(x, y, z, sm.lut1, sm.cell1, sm.nbx1, sm.nby1,
                                                                      sm.bnd_xi[1], thr1, lane, &dir_field, &nrm_index);
                        or_bits(sm.rec, lane, P::DIR1_BIT + (i - P::NT0) * 2 * P::BD1, 2 * P::BD1, dir_field);
                        or_bits(sm.rec, lane, P::NRM1_BIT + (i - P::NT0) * P::BN1, P::BN1, nrm_index);
                        if constexpr (QJL) { nhat = dir_lookup<P::BD1, REP>(sm.lut1, dir_field, lane); rho = sm.c_rho[1][nrm_index]; }
                    }
                }
                if constexpr (QJL) {
                    // r = u - rho^ n^ in place; the padded coordinates of the last triplet stay out of it
                    const float r0 = x - rho * nhat.x, r1 = y - rho * nhat.y, r2 = z - rho * nhat.z;
                    sm.u[3 * i][lane] = r0;
                    rsq = fmaf(r0, r0, rsq);
                    if (3 * i + 1 < D) { sm.u[3 * i + 1][lane] = r1; rsq = fmaf(r1, r1, rsq); }
                    if (3 * i + 2 < D) { sm.u[3 * i + 2][lane] = r2; rsq = fmaf(r2, r2, rsq); }
                }
            }
            if constexpr (QJL) sm.res_sq[wave][lane] = rsq;
        }
        __syncthreads();

        // E8: store the tile, 16 bytes per (granule, key), coalesced over keys
        // pt.table (or NULL): `cache` is a pool of [page][KV head] tiles, logical tile j of sequence s is in page
        // pt.table[s * pt.stride + j] (clamped to the pool)
        uint4 *dst = region + tile * (P::GRANULES * kWave);
        if (pt.table != nullptr) {
            const int page = page_asked;
            dst = cache + (static_cast<int64_t>(min(max(page, 0), pt.n_pages - 1)) * n_kv_heads + kvh) * (P::GRANULES * kWave);
        }
        for (int e = tid; e < P::GRANULES * kWave; e += NT) {
            const int g = e / kWave, key = e % kWave;
            const int64_t tok = tile * kWave + key;
            if (tok >= tok_lo && tok < tok_hi) {
                // non-temporal: the records are not read again by this kernel, and lines left behind in the caches
                // (dirty, a whole prefill's worth) slow down whatever streams through memory next
                typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                const u32x4_t rec4 = {sm.rec[4 * g][key], sm.rec[4 * g + 1][key], sm.rec[4 * g + 2][key],
                                      sm.rec[4 * g + 3][key]};
                __builtin_nontemporal_store(rec4, reinterpret_cast<u32x4_t *>(dst + e));
            }
        }

        if constexpr (QJL) {
            // sigma = sign(H diag(s2) r): the same two radix passes, signs applied on the way in, no scaling
            constexpr int R2 = D / 16;
            for (int g = wave; g < D / 16; g += NWV) {
                const uint32_t sb = signs2[kvh * (D / 8) + 2 * g] | (static_cast<uint32_t>(signs2[kvh * (D / 8) + 2 * g + 1]) << 8);
                float x[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float val = sm.u[g * 16 + e][lane];
                    x[e] = ((sb >> e) & 1u) ? -val : val;
                }
                butterflies<16>(x);
#pragma unroll
                for (int e = 0; e < 16; ++e) sm.u[g * 16 + e][lane] = x[e];
            }
            __syncthreads();
            for (int lo = wave; lo < 16; lo += NWV) {
                float x[R2];
#pragma unroll
                for (int e = 0; e < R2; ++e) x[e] = sm.u[e * 16 + lo][lane];
                butterflies<R2>(x);
#pragma unroll
                for (int e = 0; e < R2; ++e) sm.u[e * 16 + lo][lane] = x[e];
            }
            __syncthreads();
            constexpr int TQ = kWave * (D / 8 + 2);   // side-car bytes per tile
            unsigned char *qt = qjl + ((static_cast<int64_t>(seq) * n_kv_heads + kvh) * (t_capacity / kWave) + tile) * TQ;
            if (pt.table != nullptr) {   // the side-car in pages: a pool of [page][KV head] tiles, like the keys'
                const int page = page_asked;
                qt = qjl + (static_cast<int64_t>(min(max(page, 0), pt.n_pages - 1)) * n_kv_heads + kvh) * TQ;
            }
            const int64_t tok = tile * kWave + lane;
            const bool valid = tok >= tok_lo && tok < tok_hi;
            for (int wd = wave; wd < D / 32; wd += NWV) {
                uint32_t bits = 0u;
#pragma unroll
                for (int e = 0; e < 32; ++e) bits |= (sm.u[32 * wd + e][lane] < 0.0f ? 1u : 0u) << e;
                if (valid) reinterpret_cast<uint32_t *>(qt)[wd * kWave + lane] = bits;
            }
            if (wave == 0 && valid) {
                float n2 = 0.0f;
#pragma unroll
                for (int wv = 0; wv < NWV; wv += 4)
                    n2 += (sm.res_sq[wv][lane] + sm.res_sq[wv + 1][lane]) + (sm.res_sq[wv + 2][lane] + sm.res_sq[wv + 3][lane]);
                reinterpret_cast<__half *>(qt + (D / 8) * kWave)[lane] = __float2half_rn(sqrtf(n2));
            }
        }
    }
}

template <class P>
int launch_encode_plan(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                       int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                       const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                       const uint8_t *signs2, void *qjl, hipStream_t stream, PageTable pt = PageTable{nullptr, 0, 0}) {
    const DeviceBooks books = device_books(cb);
    // a start that is not a multiple of 64 makes the new tokens straddle one more tile
    const int tiles = (n_new + kWave - 1) / kWave + (start_pos ? 1 : 0);
    const int tpg = encode_tiles_per_group(tiles, n_kv_heads, n_seq);
    const dim3 grid((tiles + tpg - 1) / tpg, n_kv_heads, n_seq);
    const bool bf16 = key_dtype == OCTOPUS_DTYPE_BF16;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(encode_threads<P>()), 0, stream, books, keys, stride_seq, stride_tok, stride_head, n_new,
                           signs, static_cast<uint4 *>(cache), t_capacity, start_pos, n_kv_heads, signs2,
                           static_cast<unsigned char *>(qjl), 1, pt, tpg);
    };
    if (qjl != nullptr) {
        if (bf16) go(encode_kernel<P, true, true>); else go(encode_kernel<P, false, true>);
    } else {
        if (bf16) go(encode_kernel<P, true, false>); else go(encode_kernel<P, false, false>);
    }
    return static_cast<int>(hipGetLastError());
}

// The default encoder alone (local 3x3, no side-car, no pages): what the pairs of the App. D sweep are built with.
template <class P>
int launch_encode_basic_plan(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                             int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                             const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                             hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    const int tiles = (n_new + kWave - 1) / kWave + (start_pos ? 1 : 0);
    const int tpg = encode_tiles_per_group(tiles, n_kv_heads, n_seq);
    const dim3 grid((tiles + tpg - 1) / tpg, n_kv_heads, n_seq);
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(encode_threads<P>()), 0, stream, books, keys, stride_seq, stride_tok, stride_head, n_new,
                           signs, static_cast<uint4 *>(cache), t_capacity, start_pos, n_kv_heads, nullptr, nullptr, 1,
                           PageTable{nullptr, 0, 0}, tpg);
    };
    if (key_dtype == OCTOPUS_DTYPE_BF16) go(encode_kernel<P, true, false>);
    else go(encode_kernel<P, false, false>);
    return static_cast<int>(hipGetLastError());
}

// The encoder with the rounding mode chosen at run time (no side-car).
template <class P>
int launch_encode_rounding_plan(const octopus_codebooks_t &cb, const void *keys, int key_dtype, int64_t stride_seq,
                                int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads,
                                int32_t n_new, const uint8_t *signs, void *cache, int64_t t_capacity,
                                const int32_t *start_pos, int32_t mode, hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    const int tiles = (n_new + kWave - 1) / kWave + (start_pos ? 1 : 0);
    const int tpg = encode_tiles_per_group(tiles, n_kv_heads, n_seq);
    const dim3 grid((tiles + tpg - 1) / tpg, n_kv_heads, n_seq);
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(encode_threads<P>()), 0, stream, books, keys, stride_seq, stride_tok, stride_head, n_new,
                           signs, static_cast<uint4 *>(cache), t_capacity, start_pos, n_kv_heads, nullptr, nullptr, mode,
                           PageTable{nullptr, 0, 0}, tpg);
    };
    if (key_dtype == OCTOPUS_DTYPE_BF16) go(encode_kernel<P, true, false, true>);
    else go(encode_kernel<P, false, false, true>);
    return static_cast<int>(hipGetLastError());
}

}  // namespace octopus

#endif
