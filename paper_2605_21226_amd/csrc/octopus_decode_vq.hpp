// Fused decode attention over compressed keys AND group-quantised values with P.V on the matrix cores
// (Alg. 2 with its "value dequantization" step; value format of Sec. 4, "value-side group size").
#ifndef OCTOPUS_DECODE_VQ_HPP_
#define OCTOPUS_DECODE_VQ_HPP_

#include "octopus_decode.hpp"

namespace octopus {

// A value row is [v_bits-bit codes, channel j at bit v_bits * j][per group of v_group channels: fp32 scale,
// fp32 zero point] and stands for zero + scale * code.  Hence, for a query row with probabilities p_t,
//   out[ch] = sum_t (p_t scale_t[g(ch)]) (B + code_t[ch])  +  sum_t p_t (zero_t[g(ch)] - B scale_t[g(ch)])
// for any constant B: the first sum is a dense product whose right operand is made of small integers, exact
// in bf16, and whose left operand is the probability row scaled per group of channels; the second needs one
// number per (row, group).  The matrix cores take the first: v_mfma_f32_16x16x32_bf16 with M = (group, row,
// leading part / remainder), K = keys, N = channels.  Nothing is dequantised element by element, and with
// B = 2^v_bits no code is even converted: the bf16 number B + code is a constant exponent with the code in the
// top v_bits bits of the mantissa, i.e. the code bits shifted into place under a constant.
//
//   * the wavefront copies a step's rows as they lie in memory (16 bytes per lane and load, whole cache
//     lines per instruction, one step ahead of use) into LDS;
//   * after the softmax lane = key holds its probabilities; it reads the scales and zero points of ITS row,
//     adds its share of the second sum to per-lane accumulators (reduced over the wave once per work item)
//     and writes the products p scale, split into two bf16 numbers (nearest, then the remainder), to LDS in
//     the order the A operands want them: [group][part][row][key slot];
//   * lane (n, g) of the MFMA owns, of every 64-channel piece of a row, the four channels 4 n .. 4 n + 3:
//     4 v_bits bits, which it cuts out of LDS for its 8 keys of a k-step; two keys' fields side by side in
//     one register yield a word of any of the four B operands with one shift and one and-or;
//   * N-block c of piece c / 4 is the channel set {64 (c / 4) + 4 n + c % 4}; its 16 columns span
//     64 / v_group groups, 16 / (64 / v_group) adjacent columns each;
//   * an A operand stacks the rows of GPA groups (two when there are at most four query rows, else one),
//     leading parts in rows r, remainders in rows RP + r of the group's share; a column reads the rows of ITS
//     group from the result and ignores the others, so an N-block costs NA = (64 / v_group) / GPA MFMAs per
//     k-step: one for groups of 32 channels and four query rows, the same as over bf16 values.
constexpr int kVqRow = kWave + 8;   // uint16 per row of scaled probabilities in LDS

template <class P, int RG, int VB, int VG, int NW>
struct VqGeometryN {
    static constexpr int D = P::D;
    static constexpr int KPL = 1;                           // tiles per step: one key per lane
    static constexpr int NWV = NW;                          // wavefronts per workgroup
    static constexpr int CB = VB * D / 8;                   // code bytes per row
    static constexpr int G = D / VG;                        // groups per row
    static constexpr int RB = CB + 8 * G;                   // bytes per row
    static constexpr int STEP_BYTES = KPL * kWave * RB;     // the rows of a step are contiguous
    static constexpr int NLS = (STEP_BYTES + 1023) / 1024;  // 16-byte loads per lane and step
    static constexpr int PCS = D / 64;                      // 64-channel pieces of a row
    static constexpr int CPL = D / 16;                      // N-blocks
    static constexpr int RP = RG <= 4 ? 4 : 8;
    static constexpr int GPB = 64 / VG;                     // groups per piece = per N-block
    static constexpr int GPA = RP == 4 ? 2 : 1;             // groups per A operand
    static constexpr int NA = GPB / GPA;                    // A operands per piece = accumulators per N-block
    static constexpr int ZP = RG * G;                       // (row, group) pairs of the zero-point sums
};

template <class P, int RG, int VB, int VG, int NW>
struct DecodeSmemVqN {
    using Gm = VqGeometryN<P, RG, VB, VG, NW>;
    DecodeTables<P> tb;
    // scaled probabilities of a 64-key tile as bf16: [group][leading part, remainder][row][key slot];
    // a row is padded by 16 bytes, so that the 16 rows the lanes of an A operand read lie in different banks
    __attribute__((aligned(16))) uint16_t xs[Gm::NWV][Gm::G][2][RG][kVqRow];
    float zbuf[Gm::NWV][Gm::ZP];
    __attribute__((aligned(16))) unsigned char stage[Gm::NWV][Gm::STEP_BYTES];
};

template <class P, int RG, int VB, int VG, int NW>
constexpr bool vq_lds_fits_n() {
    return sizeof(DecodeSmemVqN<P, RG, VB, VG, NW>) + (mx_scores<P>() ? sizeof(QueryOperands<P, RG>) : 16) + 64 <= 160 * 1024;
}

// Wavefronts per workgroup: two per SIMD up to d = 128 (each within 256 registers), whose different phases --
// vector work, matrix-core work, LDS traffic -- the hardware overlaps, where the LDS of eight wavefronts fits (each
// has its own staging buffer and probability rows) and the kernel fits 256 registers: up to 8 accumulator tiles
// (with 16 it spills, and one wavefront per SIMD with 512 registers is faster: row groups of eight at d = 128
// 0.42 -> 0.33 ms, groups of 16 channels 0.30 -> 0.24 ms on the Llama-shaped batch); else, and at d = 256, one per
// SIMD.
template <class P, int RG, int VB, int VG>
constexpr int vq_waves() {
    using G8 = VqGeometryN<P, RG, VB, VG, 8>;
    return (P::D <= 128 && G8::CPL * G8::NA <= 8 && vq_lds_fits_n<P, RG, VB, VG, 8>()) ? 8 : 4;
}

template <class P, int RG, int VB, int VG>
using VqGeometry = VqGeometryN<P, RG, VB, VG, vq_waves<P, RG, VB, VG>()>;
template <class P, int RG, int VB, int VG>
using DecodeSmemVq = DecodeSmemVqN<P, RG, VB, VG, vq_waves<P, RG, VB, VG>()>;

// Shapes the kernel is built for: row groups of 4 or 8, at most 64 (row, group) pairs, at most 32
// accumulator tiles, everything within the 160 KB of LDS.
template <class P, int RG, int VB, int VG>
constexpr bool vq_lds_fits() { return vq_lds_fits_n<P, RG, VB, VG, vq_waves<P, RG, VB, VG>()>(); }
template <class P, int RG, int VB, int VG>
constexpr bool vq_mfma_fits() {
    using Gm = VqGeometry<P, RG, VB, VG>;
    return (RG == 4 || RG == 8) && Gm::ZP <= 64 && Gm::CPL * Gm::NA <= 32 && vq_lds_fits<P, RG, VB, VG>();
}

// wavefronts per workgroup of the kernel for a shape, 0 if none is built
template <class P, int RG, int VB, int VG>
constexpr int vq_mfma_wavefronts() { return vq_mfma_fits<P, RG, VB, VG>() ? vq_waves<P, RG, VB, VG>() : 0; }

template <class P, int RG, int VB, int VG>
__global__ __launch_bounds__((vq_waves<P, RG, VB, VG>() * kWave))
    __attribute__((amdgpu_waves_per_eu(vq_waves<P, RG, VB, VG>() / 4, vq_waves<P, RG, VB, VG>() / 4))) void decode_kernel_vq_mfma(
    DeviceBooks books, DecodeShape shp, const float *__restrict__ q_rot, const uint4 *__restrict__ cache,
    const unsigned char *__restrict__ vq, const int32_t *__restrict__ seq_lens, float *__restrict__ part_ml,
    float *__restrict__ part_acc, int32_t *__restrict__ plan, PageTable pt) {
    // pt.table (or NULL): `cache` and `vq` are pools of 64-token pages, [page][KV head] each a key tile of the cache
    // layout and 64 value rows; logical tile j of sequence s lives in page pt.table[s * pt.stride + j] (ids outside
    // the pool are clamped: a wrong table reads wrong pages, never outside the pools).
    using Gm = VqGeometry<P, RG, VB, VG>;
    static_assert(RG == 4 || RG == 8, "row groups of 4 or 8");
    constexpr int D = P::D, KPL = Gm::KPL, CPL = Gm::CPL, RP = Gm::RP, RB = Gm::RB, CB = Gm::CB;
    constexpr int PCS = Gm::PCS, NA = Gm::NA, GPA = Gm::GPA, GPB = Gm::GPB, G = Gm::G, NLS = Gm::NLS, NWV = Gm::NWV;
    constexpr int STEP_BYTES = Gm::STEP_BYTES;
    constexpr int TILEB = P::GRANULES * kWave * 16;  // bytes per cache tile
    constexpr bool MX = mx_scores<P>();
    // bf16 of 2^VB + code: exponent 127 + VB, the code in the top VB bits of the 7-bit mantissa
    constexpr float BIAS = static_cast<float>(1 << VB);
    constexpr int CODE_POS = 7 - VB;
    constexpr uint32_t CODE_MASK = (((1u << VB) - 1u) << CODE_POS) * 0x00010001u;
    constexpr uint32_t CODE_BASE = (static_cast<uint32_t>(127 + VB) << 7) * 0x00010001u;
    constexpr int KS = 2 * KPL;
    __shared__ DecodeSmemVq<P, RG, VB, VG> sm;
    __shared__ __attribute__((aligned(16))) uint4 qop_store[MX ? P::NTRI * QueryOperands<P, RG>::ROWS : 1];
    const QueryOperands<P, RG> &qop = *reinterpret_cast<const QueryOperands<P, RG> *>(&qop_store[0]);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    bool tables_built = false;
    __shared__ int item_slot;
    WaveWork ww;
    const float *qg = q_rot;
    const char *k_region = reinterpret_cast<const char *>(cache);
    const char *v_pair = reinterpret_cast<const char *>(vq);
    const int n16 = lane & 15, g4 = lane >> 4;
    const uint32_t k_lane = lane * 16u;
    const int ppos = (lane & 32) + 8 * (lane & 3) + ((lane & 31) >> 2);  // slot of key `lane` in a probability row

    // ---- per-lane LDS addresses; everything else is an immediate offset -----------------------------------
    unsigned char *stage_w = &sm.stage[wave][0];
    // k-slot j of k-step ks is, for this lane, row 32 ks + 4 j + g4 of the step.
    // A operand row of this lane: query row a_r, leading part or remainder, first or second group of the operand
    const int a_r = n16 & (RP - 1);
    const int a_part = RP == 4 ? (n16 >> 2) & 1 : n16 >> 3;
    const int a_member = RP == 4 ? (n16 >> 3) : 0;
    const uint16_t *xs_lane = &sm.xs[wave][a_member][a_part][a_r][8 * g4];
    // the four channels 4 n16 .. + 3 of a piece: 4 VB bits at bit 4 VB n16 of the piece's 8 VB bytes
    constexpr int PIECE_BYTES = 8 * VB;
    const int code_bit = 4 * VB * n16;
    const unsigned char *code_lane = stage_w + g4 * RB + (VB == 3 ? (code_bit >> 5) * 4 : (code_bit >> 3));
    const uint32_t code_sh = static_cast<uint32_t>(code_bit & 31);
    // producer side: lane = key of a tile
    const unsigned char *meta_lane = stage_w + lane * RB + CB;
    uint16_t *xs_key = &sm.xs[wave][0][0][0][ppos];

    const bool paged = pt.table != nullptr;
    // The page of a step's tile is read one step before the step's loads are issued, through the vector memory path
    // (every lane the same entry), so that nothing waits for the table right after asking it.
    int lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    auto page_ask = [&](int step) -> int {
        const int tile = max(min(step * KPL, ww.n_tiles - 1), 0);
        return pt.table[static_cast<int64_t>(ww.seq) * pt.stride + tile + lane_zero];
    };
    // position of a page's tile of this item's KV head in the pools, in tiles
    auto page_slot = [&](int asked) -> int64_t {
        const int id = __builtin_amdgcn_readfirstlane(asked);
        return static_cast<int64_t>(min(max(id, 0), pt.n_pages - 1)) * shp.n_kv_heads + ww.kvh;
    };
    auto load_record = [&](const char *src, uint32_t (&w)[P::NWORDS]) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
        typedef const u32x4_t __attribute__((address_space(1))) *g4_t;
        typedef const u32x3_t __attribute__((address_space(1))) *g3_t;
        typedef const u32x2_t __attribute__((address_space(1))) *g2_t;
        typedef const uint32_t __attribute__((address_space(1))) *g1_t;
        constexpr int USED = (P::RECORD_BYTES + 3) / 4;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            const char *gp = src + g * (kWave * 16) + k_lane;
            const int n = (USED - 4 * g) < 4 ? (USED - 4 * g) : 4;
            if (n == 4) {
                const u32x4_t x = __builtin_nontemporal_load((g4_t)(gp));
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = x.w;
            } else if (n == 3) {
                const u32x3_t x = __builtin_nontemporal_load((g3_t)(gp));
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = 0u;
            } else if (n == 2) {
                const u32x2_t x = __builtin_nontemporal_load((g2_t)(gp));
                w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = 0u; w[4 * g + 3] = 0u;
            } else {
                w[4 * g] = __builtin_nontemporal_load((g1_t)(gp));
                w[4 * g + 1] = 0u; w[4 * g + 2] = 0u; w[4 * g + 3] = 0u;
            }
        }
    };
    // slot: the pool position of the step's tile (paged cache only)
    auto load_records = [&](int step, int64_t slot, uint32_t (&w)[KPL][P::NWORDS]) {
        static_assert(KPL == 1, "one tile per step");
        const int64_t tile = paged ? slot : static_cast<int64_t>(min(step * KPL, ww.n_tiles - 1));
        load_record(k_region + tile * TILEB, w[0]);
    };
    // The value rows of a step come through a buffer descriptor that ends with the sequence's last token (rows
    // past it read as zeros: code 0, scale 0, zero point 0); the descriptor of a step that does not exist is
    // empty and its loads move nothing.  Streamed data: non-temporal.
    auto load_rows = [&](int step, int64_t slot, bool exists, uint4 (&rows)[NLS]) {
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
        const int t0 = step * (KPL * kWave);
        const int n_valid = exists ? min(KPL * kWave, ww.len - t0) : 0;
        const int64_t first_row = paged ? slot * kWave : static_cast<int64_t>(t0);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(v_pair + first_row * RB), 0, n_valid * RB, 0x00020000);
#pragma unroll
        for (int i = 0; i < NLS; ++i) {
            const u32x4_t x = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (i * kWave + lane) * 16, 0, kStreamPolicy);
            rows[i] = make_uint4(x.x, x.y, x.z, x.w);
        }
    };

    float m_run[RG], l_lane[RG], zacc[RG][G];
    f32x4_t acc[CPL][NA];

    // Producer of tile k: scaled probabilities to LDS, zero-point sums to registers.
    auto load_meta = [&](float2 (&sz)[KPL][G]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < KPL; ++k)
#pragma unroll
            for (int g = 0; g < G; ++g) sz[k][g] = *reinterpret_cast<const float2 *>(meta_lane + (k * kWave) * RB + 8 * g);
    };
    auto produce = [&](auto kk, const float (&p)[KPL][RG], const float2 (&sz)[KPL][G]) __attribute__((always_inline)) {
        constexpr int k = decltype(kk)::value;
        uint16_t *dst = xs_key;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float zero_b = fmaf(-BIAS, sz[k][g].x, sz[k][g].y);
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const float x = p[k][r] * sz[k][g].x;
                const uint32_t xr = __float_as_uint(x) + 0x8000u;   // nearest (ties up): the remainder has either sign
                const float rem = x - __uint_as_float(xr & 0xffff0000u);
                dst[((g * 2 + 0) * RG + r) * kVqRow] = static_cast<uint16_t>(xr >> 16);
                dst[((g * 2 + 1) * RG + r) * kVqRow] = static_cast<uint16_t>(__float_as_uint(rem) >> 16);
                zacc[r][g] = fmaf(p[k][r], zero_b, zacc[r][g]);
            }
        }
    };
    // The B operands of a step are built during its score pass, half a piece = (k-step, 64-channel piece of the
    // rows, 4 of the lane's 8 keys) at a time, from the staged rows alone (the pass keeps the matrix cores and LDS busy and leaves the
    // vector units idle; building the operands is vector work).  The words around the code fields of a piece
    // are requested one slot before they are used.
    constexpr int NPB = 2 * KS * PCS;   // half pieces: 4 keys (2 words of each of the piece's 4 B operands) each
    struct RawPiece { uint32_t lo[4], hi[4]; };
    RawPiece raw[NPB];
    uint32_t vbw[KS][PCS][4][4];   // [k-step][piece][N-block of the piece][word]
    auto raw_request = [&](auto pp) __attribute__((always_inline)) {
        constexpr int pi = decltype(pp)::value, ks = pi / (2 * PCS), pc = (pi / 2) % PCS, half = pi % 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned char *src = code_lane + (32 * ks + 4 * (4 * half + j)) * RB + pc * PIECE_BYTES;
            if constexpr (VB == 3) {
                const uint32_t *wp = reinterpret_cast<const uint32_t *>(src);
                raw[pi].lo[j] = wp[0];
                raw[pi].hi[j] = wp[1];
            } else if constexpr (VB == 4) {
                raw[pi].lo[j] = *reinterpret_cast<const uint16_t *>(src);
            } else {
                raw[pi].lo[j] = *src;
            }
        }
    };
    auto b_build = [&](auto pp) __attribute__((always_inline)) {
        constexpr int pi = decltype(pp)::value, ks = pi / (2 * PCS), pc = (pi / 2) % PCS, half = pi % 2;
#pragma unroll
        for (int jh = 0; jh < 2; ++jh) {
            uint32_t t[2];
#pragma unroll
            for (int o = 0; o < 2; ++o) {
                if constexpr (VB == 3) t[o] = __builtin_amdgcn_alignbit(raw[pi].hi[2 * jh + o], raw[pi].lo[2 * jh + o], code_sh);
                else t[o] = raw[pi].lo[2 * jh + o];
            }
            const uint32_t cu = __builtin_amdgcn_perm(t[1], t[0], 0x05040100u);   // two keys' fields side by side
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int sh = CODE_POS - VB * e;   // (compile-time after unrolling)
                const uint32_t moved = sh >= 0 ? cu << sh : cu >> (-sh);
                // (written out: the compiler's own choice is an and and an or)
                uint32_t word;
                asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(word) : "v"(moved), "s"(CODE_MASK), "v"(CODE_BASE));
                vbw[ks][pc][e][2 * half + jh] = word;
            }
        }
    };
    // D6 of the step's tile: all A operands are requested, then the products run
    auto pv_tile = [&]() __attribute__((always_inline)) {
        uint4 aop[KS][PCS][NA];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int pc = 0; pc < PCS; ++pc)
#pragma unroll
                for (int a = 0; a < NA; ++a)
                    aop[ks][pc][a] = *reinterpret_cast<const uint4 *>(xs_lane + ((pc * GPB + a * GPA) * 2 * RG) * kVqRow +
                                                                      32 * ks);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int pc = 0; pc < PCS; ++pc)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    union { uint32_t u[4]; bf16x8_t b; } vb;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) vb.u[jj] = vbw[ks][pc][e][jj];
#pragma unroll
                    for (int a = 0; a < NA; ++a) {
                        union { uint4 q; bf16x8_t b; } pa;
                        pa.q = aop[ks][pc][a];
                        acc[4 * pc + e][a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.b, vb.b, acc[4 * pc + e][a], 0, 0, 0);
                    }
                }
    };

    uint4 rows[NLS];   // the value rows of the wave's next step, in flight; staged at the top of that step
    uint32_t w[KPL][P::NWORDS];   // the records of the wave's next step, in flight; replaced after the score pass
    int64_t slot_nx = 0;          // paged cache: pool position of the next step's tile
    int page_asked = 0;           // ... and the table entry of the step after it, on its way
    auto process_step = [&](int step) __attribute__((always_inline)) {
        const int t0 = step * (KPL * kWave);
        const int n_valid = min(KPL * kWave, ww.len - t0);
        // this step's rows, asked for one step ago, into LDS as they lie in memory ...
#pragma unroll
        for (int i = 0; i < NLS; ++i) {
            const int off = (i * kWave + lane) * 16;
            if ((i + 1) * 1024 <= STEP_BYTES || off < STEP_BYTES) *reinterpret_cast<uint4 *>(stage_w + off) = rows[i];
        }
        // ... and the next step's rows on their way (the row loads of a step that does not exist go through an
        // empty descriptor)
        const int step_nx = min(step + ww.step_stride, ww.step_last);
        if (paged) {
            slot_nx = page_slot(page_asked);
            page_asked = page_ask(min(step_nx + ww.step_stride, ww.step_last));   // used one step from here
        }
        load_rows(step_nx, slot_nx, step + ww.step_stride < ww.step_end, rows);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float s[KPL][RG];
        int q_off = 0;
        asm volatile("" : "+s"(q_off));
        // D2-D4 with the B operands of D6 built alongside: piece i is requested in chunk i (NCH - 1) / NPB of
        // the pass and built in the chunk the next piece is requested in (the last one in the last chunk)
        constexpr int NCH = score_chunks<P, RG>();
        static_assert(NCH > NPB, "a chunk of the score pass per operand piece");
        auto build_in_chunk = [&](auto cc) __attribute__((always_inline)) {
            constexpr int ci = decltype(cc)::value;
            static_for<0, NPB>([&](auto pp) {
                constexpr int pi = decltype(pp)::value;
                constexpr int built_in = pi + 1 < NPB ? (pi + 1) * (NCH - 1) / NPB : NCH - 1;
                if constexpr (built_in == ci) b_build(pp);
            });
            static_for<0, NPB>([&](auto pp) {
                constexpr int pi = decltype(pp)::value;
                if constexpr (pi * (NCH - 1) / NPB == ci) raw_request(pp);
            });
        };
        if constexpr (MX) tile_scores_mx<P, RG, KPL, decltype(build_in_chunk), (NWV > 4 ? 2 : 4)>(w, qop, sm.tb, lane, s, build_in_chunk);
        else tile_scores<P, RG, KPL>(w, qg + q_off, sm.tb, lane, s, build_in_chunk);
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const float gamma = __uint_as_float(w[k][0]);
            const bool valid = k * kWave + lane < n_valid;
#pragma unroll
            for (int r = 0; r < RG; ++r) s[k][r] = valid ? s[k][r] * gamma : -INFINITY;
        }
        // the records are used up: the next step's take their place (the wave's last step re-reads its own);
        // scales and zero points of this lane's keys for the products below
        load_records(step_nx, slot_nx, w);
        float2 sz[KPL][G];
        load_meta(sz);
        // D5: online softmax, one running maximum per row for the whole wave; s becomes the probabilities
        float alpha[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            float mx = s[0][r];
#pragma unroll
            for (int k = 1; k < KPL; ++k) mx = fmaxf(mx, s[k][r]);
            const float m_new = fmaxf(m_run[r], wave_max(mx));
            alpha[r] = exp2_raw((m_run[r] - m_new) * kLog2e);
            m_run[r] = m_new;
            float psum = 0.0f;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                s[k][r] = exp2_raw((s[k][r] - m_new) * kLog2e);
                psum += s[k][r];
            }
            l_lane[r] = fmaf(l_lane[r], alpha[r], psum);
        }
        // the running sums are rescaled only when a row's maximum has moved (rare after a sequence's first steps)
        bool moved = false;
#pragma unroll
        for (int r = 0; r < RG; ++r) moved |= alpha[r] != 1.0f;
        if (__builtin_amdgcn_readfirstlane(moved)) {
#pragma unroll
            for (int r = 0; r < RG; ++r)
#pragma unroll
                for (int g = 0; g < G; ++g) zacc[r][g] *= alpha[r];
            // accumulator rows of this lane: m = 4 g4 + i, query row m % RP
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float a;
                if constexpr (RP == 4) a = alpha[i];
                else a = (g4 & 1) ? alpha[4 + i] : alpha[i];
#pragma unroll
                for (int c = 0; c < CPL; ++c)
#pragma unroll
                    for (int hh = 0; hh < NA; ++hh) acc[c][hh][i] *= a;
            }
        }
        // D6: the tile's scaled probabilities go to LDS, then its two k-steps run
        static_assert(KPL == 1, "one tile per step");
        produce(std::integral_constant<int, 0>{}, s, sz);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        pv_tile();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    int it, taken = 0;
    while (next_item(plan, &item_slot, tid, &taken, &it)) {
        item_work(shp, plan, seq_lens, it, wave, KPL, &ww);
        qg = q_rot + ww.group_id * (P::QS * RG);
        k_region = reinterpret_cast<const char *>(cache) + (paged ? 0 : ww.pair * shp.t_capacity * (P::GRANULES * 16));
        v_pair = reinterpret_cast<const char *>(vq) + (paged ? 0 : ww.pair * shp.t_capacity * RB);
        {   // the record pointer loses its "read-only" provenance: see decode_kernel_mfma
            const uint64_t bits = reinterpret_cast<uint64_t>(k_region);
            uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits));
            uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits >> 32));
            asm volatile("" : "+s"(lo), "+s"(hi));
            k_region = reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
        }
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            m_run[r] = -INFINITY;
            l_lane[r] = 0.0f;
#pragma unroll
            for (int g = 0; g < G; ++g) zacc[r][g] = 0.0f;
        }
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int hh = 0; hh < NA; ++hh) acc[c][hh] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

        const bool any = ww.step_begin < ww.step_end;
        int64_t slot_first = 0;
        if (paged && any) {
            slot_first = page_slot(page_ask(ww.step_begin));
            page_asked = page_ask(min(ww.step_begin + ww.step_stride, ww.step_last));
        }
        if (any) load_records(ww.step_begin, slot_first, w);
        load_rows(ww.step_begin, slot_first, any, rows);
        if (!tables_built) {   // workgroup-uniform
            build_tables<P, MX>(sm.tb, books, tid, NWV * kWave);
            tables_built = true;
        }
        if constexpr (MX) {
            // The item's rotated queries as matrix-core operands.  Every wavefront is past the previous item
            // here (next_item's barriers, or this is the workgroup's only item).
            constexpr int ROWS = QueryOperands<P, RG>::ROWS;
            uint4 *dst = reinterpret_cast<uint4 *>(&qop_store[0]);
            for (int e = tid; e < P::NTRI * ROWS; e += NWV * kWave) {
                const int i = e / ROWS, r = e % ROWS;
                float x = 0.0f, y = 0.0f, z = 0.0f;
                if (r < RG) {
                    x = qg[(3 * i) * RG + r];
                    y = qg[(3 * i + 1) * RG + r];
                    z = qg[(3 * i + 2) * RG + r];
                }
                dst[e] = split_triplet(x, y, z);
            }
            __syncthreads();
        }
        for (int step = ww.step_begin; step < ww.step_end; step += ww.step_stride) process_step(step);

        // D7: the zero-point sums of the lanes are added up and handed to the lanes that hold the channels ...
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float z = wave_sum(zacc[r][g]);
                if (lane == 0) sm.zbuf[wave][g * RG + r] = z;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // ... which add the leading-part and remainder rows of their group (lane groups 16 or 32 lanes apart)
        // and emit the wave's partial of this item
        const int64_t pbase = (static_cast<int64_t>(it) * NWV + wave) * RG;
        const int lgrp = (4 * n16) / VG;                 // group of this lane's columns within a piece
        const int a_sel = lgrp / GPA, member = lgrp % GPA;
        const bool holder = RP == 4 ? g4 == 2 * member : g4 < 2;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const int channel = 64 * (c / 4) + 4 * n16 + c % 4;
            const int group = (c / 4) * GPB + lgrp;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float tot = 0.0f;
#pragma unroll
                for (int hh = 0; hh < NA; ++hh) {
                    const float t = acc[c][hh][i] + __shfl_down(acc[c][hh][i], RP * 4, kWave);
                    tot = a_sel == hh ? t : tot;
                }
                const int r = RP == 4 ? i : 4 * g4 + i;
                if (holder && ww.grp * RG + r < shp.rows_per_kv)
                    part_acc[(pbase + r) * D + channel] = tot + sm.zbuf[wave][group * RG + (r & (RG - 1))];
            }
        }
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const float l = wave_sum(l_lane[r]);
            if (lane == 0) {
                part_ml[(pbase + r) * 2] = m_run[r];
                part_ml[(pbase + r) * 2 + 1] = l;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// -1: no kernel for this shape (the caller falls back to the vector-unit kernel).
template <class P, int RG, int VB, int VG>
int launch_decode_vq_mfma_one(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                              const void *vq, const int32_t *seq_lens, float *part_ml, float *part_acc, int32_t *plan,
                              hipStream_t stream, const PageTable &pt) {
    if constexpr (vq_mfma_fits<P, RG, VB, VG>()) {
        const DeviceBooks books = device_books(cb);
        constexpr int NWV = VqGeometry<P, RG, VB, VG>::NWV;
        if (s.item_waves != NWV || s.tiles_per_step != 1) return static_cast<int>(hipErrorInvalidValue);
        hipLaunchKernelGGL((decode_kernel_vq_mfma<P, RG, VB, VG>), dim3(kDecodeWorkgroups), dim3(NWV * kWave), 0,
                           stream, books, s, q_rot, static_cast<const uint4 *>(cache),
                           static_cast<const unsigned char *>(vq), seq_lens, part_ml, part_acc, plan, pt);
        return static_cast<int>(hipGetLastError());
    } else {
        return -1;
    }
}

template <class P, int VB>
int launch_decode_vq_mfma_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                               const void *cache, const void *vq, int v_group, const int32_t *seq_lens, float *part_ml,
                               float *part_acc, int32_t *plan, hipStream_t stream, const PageTable &pt) {
    if (v_group == 32) {
        if (s.rows_per_pass == 4) return launch_decode_vq_mfma_one<P, 4, VB, 32>(cb, s, q_rot, cache, vq, seq_lens, part_ml, part_acc, plan, stream, pt);
        if (s.rows_per_pass == 8) return launch_decode_vq_mfma_one<P, 8, VB, 32>(cb, s, q_rot, cache, vq, seq_lens, part_ml, part_acc, plan, stream, pt);
    } else if (v_group == 16) {
        if (s.rows_per_pass == 4) return launch_decode_vq_mfma_one<P, 4, VB, 16>(cb, s, q_rot, cache, vq, seq_lens, part_ml, part_acc, plan, stream, pt);
        if (s.rows_per_pass == 8) return launch_decode_vq_mfma_one<P, 8, VB, 16>(cb, s, q_rot, cache, vq, seq_lens, part_ml, part_acc, plan, stream, pt);
    }
    return -1;
}

}  // namespace octopus

#endif
