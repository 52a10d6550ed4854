// Value codec: per-group uniform quantisation of value rows (Sec. 4, "value-side group size in {16, 32}").
// The paper fixes the group size, the bit width and (through the KV ratios of Table (kernel speed)) the row
// size b d / 8 + 8 d / g bytes; the codec itself is this library's reading: asymmetric min/max quantisation
// per group with an fp32 scale and an fp32 zero point.
#include <hip/hip_runtime.h>

#include "octopus_internal.h"

namespace octopus {

// Minimum / maximum of three numbers in one instruction; a quiet NaN among them is passed over.
__device__ __forceinline__ float min3_plain(float a, float b, float c) {
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max3_plain(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

constexpr int kTokenSlab = 1 << 18;   // tokens per grid y: with at most 4096 (KV head, group) pairs a token, 2^30 threads

// One thread per (token, KV head, group): min and max of the group's G values, scale = (max - min) /
// (2^B - 1), code = rint((v - min) / scale) clamped; each a single correctly rounded fp32 operation.
// VEC16: every group starts on a 16-byte boundary of the input (16-byte loads).
template <bool BF16, int B, int G>
__global__ __launch_bounds__(256) void encode_values_kernel(const void *__restrict__ v, int64_t stride_seq,
                                                             int64_t stride_tok, int64_t stride_head, int32_t n_seq,
                                                             int32_t n_kv_heads, int32_t n_new, int32_t d,
                                                             unsigned char *__restrict__ vq, int64_t t_capacity,
                                                             const int32_t *__restrict__ start_pos, int vec16,
                                                             PageTable pt) {
    constexpr int LEVELS = (1 << B) - 1;
    constexpr int CODE_WORDS = G * B / 32 + ((G * B) % 32 ? 1 : 0);   // 1, 2, 3 or 4
    constexpr int CODE_BYTES = G * B / 8;                             // the group's codes: 4 .. 16 bytes
    // One sequence per grid z, kTokenSlab tokens per grid y; within a slab a 32-bit index over (token, KV head,
    // group), groups fastest (64-bit divisions by run-time numbers would cost more than the quantisation itself).
    const int n_groups = d / G;                      // a power of two
    const uint32_t per_token = static_cast<uint32_t>(n_kv_heads * n_groups);
    const uint32_t flat = blockIdx.x * 256u + threadIdx.x;
    const uint32_t slab_tok = flat / per_token, r = flat - slab_tok * per_token;
    const int64_t tok = static_cast<int64_t>(blockIdx.y) * kTokenSlab + slab_tok;
    if (slab_tok >= static_cast<uint32_t>(kTokenSlab) || tok >= n_new) return;
    const int grp = static_cast<int>(r & static_cast<uint32_t>(n_groups - 1));
    const int kvh = static_cast<int>(r >> (31 - __builtin_clz(n_groups)));
    const int seq = blockIdx.z;
    const int64_t pos = (start_pos ? max(start_pos[seq], 0) : 0) + tok;   // (a negative position would write before vq)
    if (pos >= t_capacity) return;

    const int64_t src = seq * stride_seq + tok * stride_tok + kvh * stride_head + static_cast<int64_t>(grp) * G;
    float x[G];
    if (vec16) {
        if constexpr (BF16) {
            // (plain loads: the four of a lane share cache lines with its neighbours', and the non-temporal kind
            // fetched them once per load -- 0.49 against 0.30 ms on 4.2 M rows of 128)
            const uint4 *p4 = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(v) + src);
#pragma unroll
            for (int j = 0; j < G / 8; ++j) {
                const uint4 w = p4[j];
                const uint32_t w4[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    x[8 * j + 2 * h] = __uint_as_float(w4[h] << 16);
                    x[8 * j + 2 * h + 1] = __uint_as_float(w4[h] & 0xffff0000u);
                }
            }
        } else {
            const float4 *p4 = reinterpret_cast<const float4 *>(static_cast<const float *>(v) + src);
#pragma unroll
            for (int j = 0; j < G / 4; ++j) {
                const float4 w = p4[j];
                x[4 * j] = w.x; x[4 * j + 1] = w.y; x[4 * j + 2] = w.z; x[4 * j + 3] = w.w;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < G; ++j)
            x[j] = BF16 ? __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(v)[src + j]) << 16)
                        : static_cast<const float *>(v)[src + j];
    }
    // min and max as the scan "lo = x[j] < lo ? x[j] : lo" from x[0] defines them, taken three at a time: the scan
    // keeps the FIRST element that attains the extreme, which shows only in the sign of a zero (the minimum is
    // stored, bits and all), and a NaN in x[0] stays while one elsewhere is passed over.
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int j = 1; j + 1 < G; j += 2) {
        lo = min3_plain(lo, x[j], x[j + 1]);
        hi = max3_plain(hi, x[j], x[j + 1]);
    }
    lo = min3_plain(lo, x[G - 1], x[G - 1]);
    hi = max3_plain(hi, x[G - 1], x[G - 1]);
    if (lo == 0.0f || hi == 0.0f) {
        float zero = 0.0f;
#pragma unroll
        for (int j = G - 1; j >= 0; --j) zero = x[j] == 0.0f ? x[j] : zero;   // the first zero of the group
        lo = lo == 0.0f ? zero : lo;
        hi = hi == 0.0f ? zero : hi;
    }
    if (x[0] != x[0]) lo = hi = x[0];
    const float scale = __fdiv_rn(__fsub_rn(hi, lo), static_cast<float>(LEVELS));

    // The codes, channel j of the group at bit B * j (compile-time positions).  The code is the rounding of the
    // correctly rounded quotient (v - min) / scale.  The compiler's division is ten instructions, three of them for
    // operands near the ends of the exponent range and two for a reciprocal of the divisor that all G divisions of a
    // group share.  For a scale in [2^-100, 2^100] the remaining five are issued here directly -- the product with
    // the refined reciprocal, then twice a residual and a correction, each a fused multiply-add: the same values
    // the full sequence computes when it does not rescale, and it rescales only for operands outside such a range
    // (a numerator so small that it is denormal gives a quotient that rounds to code 0 either way).  Other scales
    // (and NaN) take the compiler's division.
    uint32_t words[CODE_WORDS];
#pragma unroll
    for (int k = 0; k < CODE_WORDS; ++k) words[k] = 0u;
    const bool live = scale > 0.0f;
    const float divisor = live ? scale : 1.0f;
    float c[G];
    if (divisor > 0x1p-100f && divisor < 0x1p100f) {
        float inv = __builtin_amdgcn_rcpf(divisor);
        inv = fmaf(fmaf(-divisor, inv, 1.0f), inv, inv);
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const float t = __fsub_rn(x[j], lo);
            float q = __fmul_rn(t, inv);
            q = fmaf(fmaf(-divisor, q, t), inv, q);
            q = fmaf(fmaf(-divisor, q, t), inv, q);
            c[j] = rintf(q);
        }
    } else {
#pragma unroll
        for (int j = 0; j < G; ++j) c[j] = rintf(__fdiv_rn(__fsub_rn(x[j], lo), divisor));
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const uint32_t code = live ? static_cast<uint32_t>(fminf(fmaxf(c[j], 0.0f), static_cast<float>(LEVELS))) : 0u;
        const int bit = B * j, wi = bit >> 5, sh = bit & 31;   // constants after unrolling
        words[wi] |= code << sh;
        if (sh + B > 32) words[wi + 1] |= code >> (32 - sh);
    }
    const int row_bytes = B * d / 8 + n_groups * 8;
    // pt.table (or NULL): vq is a pool of [page][KV head][64] rows, token t of sequence s in page
    // pt.table[s * pt.stride + t / 64] (clamped to the pool); t_capacity is then what the table addresses
    int64_t row_index = (static_cast<int64_t>(seq) * n_kv_heads + kvh) * t_capacity + pos;
    if (pt.table != nullptr) {
        const int page = pt.table[static_cast<int64_t>(seq) * pt.stride + pos / 64];
        row_index = (static_cast<int64_t>(min(max(page, 0), pt.n_pages - 1)) * n_kv_heads + kvh) * 64 + pos % 64;
    }
    unsigned char *row = vq + row_index * row_bytes;
    unsigned char *dst = row + grp * CODE_BYTES;
    if constexpr (CODE_BYTES % 4 == 0) {          // rows are multiples of 8 bytes: the group starts on a word
#pragma unroll
        for (int k = 0; k < CODE_BYTES / 4; ++k) reinterpret_cast<uint32_t *>(dst)[k] = words[k];
    } else {                                      // 16 codes of 3 bits: 6 bytes, on a 2-byte boundary
#pragma unroll
        for (int k = 0; k < CODE_BYTES / 2; ++k)
            reinterpret_cast<uint16_t *>(dst)[k] = static_cast<uint16_t>(words[k / 2] >> (16 * (k & 1)));
    }
    float2 *meta = reinterpret_cast<float2 *>(row + B * d / 8 + grp * 8);
    *meta = make_float2(scale, lo);
}

int launch_encode_values(const void *v, int v_dtype, int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                         int32_t n_seq, int32_t n_kv_heads, int32_t n_new, int32_t head_dim, int32_t bits,
                         int32_t group, void *vq, int64_t t_capacity, const int32_t *start_pos, void *stream, PageTable pt) {
    const int64_t per_token = static_cast<int64_t>(n_kv_heads) * (head_dim / group);
    if (per_token > 4096 || n_seq > 65535) return static_cast<int>(hipErrorInvalidValue);
    if (n_seq == 0 || n_new == 0) return 0;
    const int64_t slab = n_new < kTokenSlab ? n_new : kTokenSlab;
    const dim3 grid(static_cast<unsigned>((slab * per_token + 255) / 256), static_cast<unsigned>((n_new + kTokenSlab - 1) / kTokenSlab),
                    static_cast<unsigned>(n_seq));
    hipStream_t st = static_cast<hipStream_t>(stream);
    // 16-byte loads when every group starts on a 16-byte boundary
    const int64_t per16 = v_dtype == OCTOPUS_DTYPE_BF16 ? 8 : 4;
    const int vec16 = (reinterpret_cast<uintptr_t>(v) % 16 == 0 && stride_seq % per16 == 0 && stride_tok % per16 == 0 &&
                       stride_head % per16 == 0) ? 1 : 0;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(256), 0, st, v, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new,
                           head_dim, static_cast<unsigned char *>(vq), t_capacity, start_pos, vec16, pt);
    };
    const bool bf16 = v_dtype == OCTOPUS_DTYPE_BF16;
#define OCTOPUS_CASE(B, G)                                                                                          \
    if (bits == B && group == G) {                                                                                  \
        if (bf16) go(encode_values_kernel<true, B, G>); else go(encode_values_kernel<false, B, G>);                 \
        return static_cast<int>(hipGetLastError());                                                                 \
    }
    OCTOPUS_CASE(2, 16) OCTOPUS_CASE(3, 16) OCTOPUS_CASE(4, 16) OCTOPUS_CASE(2, 32) OCTOPUS_CASE(3, 32) OCTOPUS_CASE(4, 32)
#undef OCTOPUS_CASE
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace octopus
