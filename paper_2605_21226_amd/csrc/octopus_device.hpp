// Device-side building blocks shared by the encode and decode kernels (gfx950, wave64).
#ifndef OCTOPUS_DEVICE_HPP_
#define OCTOPUS_DEVICE_HPP_

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <type_traits>

#include "octopus_internal.h"

namespace octopus {

constexpr int kWave = 64;
constexpr float kEps = 1e-20f;  // clamp of both divisors in Alg. 1

constexpr int cx_gcd(int a, int b) { return b == 0 ? a : cx_gcd(b, a % b); }
constexpr int cx_stream_bytes(int n, int b) {
    return (n <= 0 || b <= 0) ? 0 : ((n + 8 / cx_gcd(b, 8) - 1) / (8 / cx_gcd(b, 8))) * ((8 / cx_gcd(b, 8)) * b / 8);
}

// Compile-time image of octopus_plan_t.  BD1 == 0 means a single class.
template <int D_, int BD0_, int BN0_, int BD1_ = 0, int BN1_ = 0>
struct PlanT {
    static constexpr int D = D_;
    static constexpr int NTRI = (D + 2) / 3;
    static constexpr int NCLASS = BD1_ > 0 ? 2 : 1;
    static constexpr int NT0 = NCLASS == 2 ? (NTRI + 1) / 2 : NTRI;
    static constexpr int NT1 = NTRI - NT0;
    static constexpr int BD0 = BD0_, BN0 = BN0_, BD1 = BD1_, BN1 = BN1_;
    static constexpr int DIR0_BYTES = cx_stream_bytes(2 * NT0, BD0);
    static constexpr int DIR1_BYTES = cx_stream_bytes(2 * NT1, BD1);
    static constexpr int NRM0_BYTES = cx_stream_bytes(NT0, BN0);
    static constexpr int NRM1_BYTES = cx_stream_bytes(NT1, BN1);
    // bit offsets of the streams from the start of the record (gamma occupies bits 0..31)
    static constexpr int DIR0_BIT = 32;
    static constexpr int DIR1_BIT = DIR0_BIT + 8 * DIR0_BYTES;
    static constexpr int NRM0_BIT = DIR1_BIT + 8 * DIR1_BYTES;
    static constexpr int NRM1_BIT = NRM0_BIT + 8 * NRM0_BYTES;
    static constexpr int RECORD_BYTES = 4 + DIR0_BYTES + DIR1_BYTES + NRM0_BYTES + NRM1_BYTES;
    static constexpr int GRANULES = (RECORD_BYTES + 15) / 16;
    static constexpr int NWORDS = GRANULES * 4;
    static constexpr int QS = (3 * NTRI + 3) & ~3;  // floats per rotated query row
    static constexpr int LUT0 = 1 << (2 * BD0);     // direction LUT entries per class
    static constexpr int LUT1 = NCLASS == 2 ? 1 << (2 * BD1) : 0;

    // per-triplet constants
    static constexpr int cls(int i) { return i < NT0 ? 0 : 1; }
    static constexpr int bdir(int i) { return cls(i) ? BD1 : BD0; }
    static constexpr int bnrm(int i) { return cls(i) ? BN1 : BN0; }
    static constexpr int dir_bit(int i) { return cls(i) ? DIR1_BIT + (i - NT0) * 2 * BD1 : DIR0_BIT + i * 2 * BD0; }
    static constexpr int nrm_bit(int i) { return cls(i) ? NRM1_BIT + (i - NT0) * BN1 : NRM0_BIT + i * BN0; }

    static bool matches(const octopus_plan_t &p) {
        if (p.head_dim != D || p.n_class != NCLASS) return false;
        if (p.b_dir[0] != BD0 || p.b_nrm[0] != BN0 || p.class_ntri[0] != NT0) return false;
        if (NCLASS == 2 && (p.b_dir[1] != BD1 || p.b_nrm[1] != BN1 || p.class_ntri[1] != NT1)) return false;
        return p.record_bytes == RECORD_BYTES && p.granules == GRANULES;
    }
};

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// NBITS-wide field at compile-time bit position BITPOS of a record held in 32-bit words.
template <int BITPOS, int NBITS, int NW>
__device__ __forceinline__ uint32_t field(const uint32_t (&w)[NW]) {
    constexpr int wi = BITPOS >> 5, sh = BITPOS & 31;
    constexpr uint32_t mask = (1u << NBITS) - 1u;
    if constexpr (sh + NBITS <= 32) {
        return (w[wi] >> sh) & mask;
    } else {
        static_assert(wi + 1 < NW, "field runs past the record");
        return ((w[wi] >> sh) | (w[wi + 1] << (32 - sh))) & mask;
    }
}

// Same for a field whose upper bits may lie past the last word of the record (they read as zero).
template <int BITPOS, int NBITS, int NW>
__device__ __forceinline__ uint32_t field_clamped(const uint32_t (&w)[NW]) {
    constexpr int wi = BITPOS >> 5, sh = BITPOS & 31;
    constexpr uint32_t mask = (1u << NBITS) - 1u;
    if constexpr (sh + NBITS <= 32 || wi + 1 >= NW) {
        return (w[wi] >> sh) & mask;
    } else {
        return ((w[wi] >> sh) | (w[wi + 1] << (32 - sh))) & mask;
    }
}

// Eq. (oct-decode): unit vector of a point of the square, sign(0) = +1.
__device__ __forceinline__ float4 oct_decode(float xi, float eta) {
    const float r = 1.0f - fabsf(xi) - fabsf(eta);
    float a = xi, b = eta;
    if (r < 0.0f) {
        a = (xi >= 0.0f ? 1.0f : -1.0f) * (1.0f - fabsf(eta));
        b = (eta >= 0.0f ? 1.0f : -1.0f) * (1.0f - fabsf(xi));
    }
    const float nn = sqrtf(a * a + b * b + r * r);
    return make_float4(a / nn, b / nn, r / nn, 0.0f);
}

// Direction table of one class: entry jx | (jy << BD) holds Oct^-1(C_xi[jx], C_xi[jy]); the entry
// index is the 2*BD-bit field of the direction stream read as one number.
template <int BD>
__device__ __forceinline__ void build_dir_lut(float4 *lut, const float *c_xi, int tid, int nthreads) {
    constexpr int K = 1 << BD;
    for (int e = tid; e < K * K; e += nthreads) lut[e] = oct_decode(c_xi[e & (K - 1)], c_xi[e >> BD]);
}

// Kernel-argument centroids to LDS with compile-time indices (every lane stores the same values).  Only the
// levels that plan P has are copied: the arrays are sized for the largest plan, and each level costs the
// copying wavefront a move and an LDS store while the rest of the workgroup waits.
template <class P>
__device__ __forceinline__ void copy_books(const DeviceBooks &books, float (*c_xi)[kMaxLevels], float (*c_rho)[kMaxLevels]) {
    constexpr int two = P::NCLASS == 2 ? 1 : 0;
    constexpr int n_xi[2] = {1 << P::BD0, two << (P::BD1 > 0 ? P::BD1 : 0)};
    // (at least two norm levels, so that the first boundary of a class is a number whatever its bit width)
    constexpr int n_rho[2] = {P::BN0 > 0 ? 1 << P::BN0 : 2, two * (P::BN1 > 0 ? 1 << P::BN1 : 2)};
#pragma unroll
    for (int c = 0; c < 2; ++c) {
#pragma unroll
        for (int k = 0; k < n_xi[c]; ++k) c_xi[c][k] = books.c_xi[c][k];
#pragma unroll
        for (int k = 0; k < n_rho[c]; ++k) c_rho[c][k] = books.c_rho[c][k];
    }
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// Wave-wide reductions on the data-parallel-primitive path (no LDS traffic): shifts within rows of 16
// lanes, then row broadcasts; lane 63 ends up with the total, which is returned wave-uniform.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_take(float v) {
    // lanes whose source lane does not exist, or whose row is masked off, keep their own value
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_take<0x111, 0xf>(v));  // row_shr:1
    v = fmaxf(v, dpp_take<0x112, 0xf>(v));  // row_shr:2
    v = fmaxf(v, dpp_take<0x114, 0xf>(v));  // row_shr:4
    v = fmaxf(v, dpp_take<0x118, 0xf>(v));  // row_shr:8
    v = fmaxf(v, dpp_take<0x142, 0xa>(v));  // row_bcast:15 into rows 1 and 3
    v = fmaxf(v, dpp_take<0x143, 0xc>(v));  // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

}  // namespace octopus

#endif
