// Fused decode attention over compressed keys (Alg. 2, Eq. (score-exact)): query rotation,
// split-K main kernels, split merge.
#ifndef OCTOPUS_DECODE_HPP_
#define OCTOPUS_DECODE_HPP_

#include "octopus_device.hpp"

namespace octopus {

constexpr float kLog2e = 1.4426950408889634f;

// 2^x as the bare v_exp_f32 (about one ulp; results below 2^-126 become zero, which is all a softmax
// weight that small is worth).  exp2f() wraps the same instruction in a range fix-up for denormal
// results that costs five more instructions per value.
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr int kDecodeWaves = 4;  // wavefronts per workgroup of the main kernels
constexpr int kStreamPolicy = 2; // cache policy of the buffer loads of streamed data: non-temporal

// ---- D1-D7: split-K main kernels --------------------------------------------------------------
// Work unit = one wavefront over a range of steps of one (sequence, KV head, row group): the wave walks
// its 64-token tiles with one key per lane (two tiles per step up to d = 128), keeps its own running
// (m, l, acc) and writes one partial per query row; nothing is shared between the waves of a workgroup
// but the LDS tables.  How the ranges are cut (items) is described with the work plan below.
//
// Per tile: the lane loads its record (16 bytes at a time, coalesced thanks to the tile-interleaved
// layout, one tile ahead of use), unpacks the code fields with compile-time shifts, looks up the
// direction (and the norm centroids, a group of codes at a time) in LDS tables and accumulates the RG
// scores against the wave-uniform rotated queries, which arrive through scalar loads.  The tables
// are replicated so that neighbouring lanes always read different LDS banks whatever their codes.
// Two kernels differ in P.V only: decode_kernel_mfma (bf16 values) feeds the probabilities to the
// matrix cores; decode_kernel_valu (fp32 values) multiplies on the vector ALUs.

// Replication of a table of `bytes` bytes: up to 8 copies within a 64 KB budget (one workgroup runs
// per compute unit and may use most of its 160 KB of LDS).
constexpr int table_rep(int bytes) {
    return bytes * 8 <= 65536 ? 8 : (bytes * 4 <= 65536 ? 4 : (bytes * 2 <= 65536 ? 2 : 1));
}

template <int BD>
struct DirTable {
    static constexpr int ENTRIES = 1 << (2 * BD);
    static constexpr int REP = table_rep(ENTRIES * 16);
    static constexpr int FLOAT4S = ENTRIES * REP;
};

// Entry e of copy r sits at float4 index e * REP + r: lanes l and l' with l % REP != l' % REP never
// share a bank, whatever e.
template <int BD>
__device__ __forceinline__ void build_dir_table(float4 *table, const float *c_xi, int tid, int nthreads) {
    using T = DirTable<BD>;
    constexpr int K = 1 << BD;
    for (int e = tid; e < T::FLOAT4S; e += nthreads) {
        const int code = e / T::REP;
        table[e] = oct_decode(c_xi[code & (K - 1)], c_xi[code >> BD]);
    }
}

// Norm codes are looked up a group at a time: NTG consecutive BN-bit indices form one table index and
// the entry holds their NTG centroids (4 one-bit codes, or 2 two- or three-bit codes, per lookup).
template <int BN>
struct RhoTable {
    static constexpr int NTG = BN == 1 ? 4 : (BN <= 3 ? 2 : 1);   // (4 bits and more: one code per lookup)
    static constexpr int BITS = BN * NTG;
    static constexpr int ENTRIES = 1 << BITS;
    static constexpr int REP = 32 / NTG;   // 8 x 16 bytes, 16 x 8 bytes or 32 x 4 bytes = all 32 banks
    static constexpr int FLOATS = ENTRIES * REP * NTG;
};

template <int BN>
__device__ __forceinline__ void build_rho_table(float *table, const float *c_rho, int tid, int nthreads) {
    using T = RhoTable<BN>;
    for (int e = tid; e < T::FLOATS; e += nthreads) {
        const int t = e % T::NTG, entry = e / (T::NTG * T::REP);
        table[e] = c_rho[(entry >> (BN * t)) & ((1 << BN) - 1)];
    }
}

// Where the direction and norm codes of a triplet together have at most 10 bits (every plan up to 3 bits
// per coordinate), one table indexed by (norm code, xi code, eta code) holds the products
// rho^ * n^ themselves: one lookup per triplet, no multiply.  Otherwise (5 + 5 + 3 bits) directions and
// norm centroids come from the two tables above.
constexpr bool joint_codes(int bd, int bn) { return 2 * bd + bn <= 10; }

// Layout [direction code][norm code][copy]: the byte offset of the entry lane l reads is
//   (direction code << CS) | (norm code << NS) | ((l % REP) << 4),
// the copies making neighbouring lanes hit different banks.  For 4 + 4 + 2 bits with 4 copies CS is 8
// and the direction code is a whole byte of the record: one byte permute puts it in place together with
// the lane part, a bit-field extract and a shift-or add the norm code -- three instructions per triplet.
template <int BD, int BN>
struct JointTable {
    static constexpr int BITS = 2 * BD + BN;
    static constexpr int ENTRIES = 1 << BITS;
    static constexpr int REP = table_rep(ENTRIES * 16);
    static constexpr int LOG_REP = REP == 8 ? 3 : (REP == 4 ? 2 : (REP == 2 ? 1 : 0));
    static constexpr int NS = 4 + LOG_REP;
    static constexpr int CS = NS + BN;
    static constexpr int FLOAT4S = ENTRIES * REP;
    static constexpr bool BYTE_CODES = (2 * BD == 8) && (CS == 8);
};

template <int BD, int BN>
__device__ __forceinline__ void build_joint_table(float4 *table, const float *c_xi, const float *c_rho, int tid,
                                                  int nthreads) {
    using T = JointTable<BD, BN>;
    constexpr int K = 1 << BD;
    for (int e = tid; e < T::ENTRIES; e += nthreads) {
        const int dir = e >> BN, nrm = e & ((1 << BN) - 1);
        const float4 n = oct_decode(c_xi[dir & (K - 1)], c_xi[dir >> BD]);
        const float rho = c_rho[nrm];
        const float4 val = make_float4(rho * n.x, rho * n.y, rho * n.z, 0.0f);
#pragma unroll
        for (int r = 0; r < T::REP; ++r) table[e * T::REP + r] = val;
    }
}

// ---- operands of the matrix-core score pass --------------------------------------------------------
// fp32 -> two bf16 numbers whose sum represents it to about 2^-17 (round to nearest even both times; the
// difference x - hi is exact in fp32).
__device__ __forceinline__ uint32_t bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
// (x, y, z) -> 16 bytes: bf16 hi of (x, y, z, 0), then bf16 lo of (x, y, z, 0): the k = 4 operand of
// v_mfma_f32_4x4x4_16b_bf16, once for the leading parts and once for the remainders.
__device__ __forceinline__ uint4 split_triplet(float x, float y, float z) {
    const uint32_t hx = bf16_rne(x), hy = bf16_rne(y), hz = bf16_rne(z);
    const uint32_t lx = bf16_rne(x - __uint_as_float(hx << 16)), ly = bf16_rne(y - __uint_as_float(hy << 16)),
                   lz = bf16_rne(z - __uint_as_float(hz << 16));
    return make_uint4(hx | (hy << 16), hz, lx | (ly << 16), lz);
}

// The joint table of a class with its entries in that form (same size and addressing as the fp32 table).
template <int BD, int BN>
__device__ __forceinline__ void build_joint_table_mx(float4 *table, const float *c_xi, const float *c_rho, int tid,
                                                     int nthreads) {
    using T = JointTable<BD, BN>;
    constexpr int K = 1 << BD;
    uint4 *out = reinterpret_cast<uint4 *>(table);
    for (int e = tid; e < T::ENTRIES; e += nthreads) {
        const int dir = e >> BN, nrm = e & ((1 << BN) - 1);
        const float4 n = oct_decode(c_xi[dir & (K - 1)], c_xi[dir >> BD]);
        const float rho = c_rho[nrm];
        const uint4 val = split_triplet(rho * n.x, rho * n.y, rho * n.z);
#pragma unroll
        for (int r = 0; r < T::REP; ++r) out[e * T::REP + r] = val;
    }
}

template <int BD, int BN>
constexpr int dir_table_float4s() {
    return joint_codes(BD, BN) ? JointTable<BD, BN>::FLOAT4S : DirTable<BD>::FLOAT4S;
}

template <class P>
struct DecodeTables {
    static constexpr bool J0 = joint_codes(P::BD0, P::BN0);
    static constexpr bool J1 = P::NCLASS == 2 && joint_codes(P::BD1, P::BN1);
    float4 dir0[dir_table_float4s<P::BD0, P::BN0>()];
    float4 dir1[P::NCLASS == 2 ? dir_table_float4s<(P::BD1 > 0 ? P::BD1 : 1), (P::BN1 > 0 ? P::BN1 : 1)>() : 1];
    __attribute__((aligned(16))) float rho0[J0 ? 4 : RhoTable<P::BN0>::FLOATS];
    __attribute__((aligned(16))) float rho1[P::NCLASS == 2 && !J1 ? RhoTable<(P::BN1 > 0 ? P::BN1 : 1)>::FLOATS : 4];
    float c_xi[2][kMaxLevels];
    float c_rho[2][kMaxLevels];
};

// Plans whose every class has a joint table (all up to 3 bits per coordinate) can score on the matrix cores.
template <class P>
constexpr bool mx_scores() { return DecodeTables<P>::J0 && (P::NCLASS == 1 || DecodeTables<P>::J1); }

// MX: joint tables hold bf16 hi / lo operands (the matrix-core score pass) instead of fp32 vectors.
template <class P, bool MX = false>
__device__ __forceinline__ void build_tables(DecodeTables<P> &tb, const DeviceBooks &books, int tid, int nthreads) {
    if (tid < kWave) copy_books<P>(books, tb.c_xi, tb.c_rho);
    __syncthreads();
    if constexpr (MX) {
        static_assert(mx_scores<P>(), "matrix-core scores need joint tables");
        build_joint_table_mx<P::BD0, P::BN0>(tb.dir0, tb.c_xi[0], tb.c_rho[0], tid, nthreads);
        if constexpr (P::NCLASS == 2) build_joint_table_mx<P::BD1, P::BN1>(tb.dir1, tb.c_xi[1], tb.c_rho[1], tid, nthreads);
        __syncthreads();
        return;
    }
    if constexpr (DecodeTables<P>::J0) {
        build_joint_table<P::BD0, P::BN0>(tb.dir0, tb.c_xi[0], tb.c_rho[0], tid, nthreads);
    } else {
        build_dir_table<P::BD0>(tb.dir0, tb.c_xi[0], tid, nthreads);
        build_rho_table<P::BN0>(tb.rho0, tb.c_rho[0], tid, nthreads);
    }
    if constexpr (P::NCLASS == 2) {
        if constexpr (DecodeTables<P>::J1) {
            build_joint_table<P::BD1, P::BN1>(tb.dir1, tb.c_xi[1], tb.c_rho[1], tid, nthreads);
        } else {
            build_dir_table<P::BD1>(tb.dir1, tb.c_xi[1], tid, nthreads);
            build_rho_table<P::BN1>(tb.rho1, tb.c_rho[1], tid, nthreads);
        }
    }
    __syncthreads();
}

// Work distribution of the split-K kernels.  The kernels are launched with one workgroup per compute
// unit; the workgroups take ITEMS from a counter until none is left.  An item is a contiguous range of
// steps (a step = tiles_per_step 64-token tiles) of one (sequence, KV head, row group); its four
// wavefronts walk that range interleaved (step_begin, step_begin + 4, ...), so that the workgroup
// streams through memory front to back, and each wavefront writes its own partial result, addressed by
// (item, wavefront).  The items are cut on the device from the actual sequence lengths (plan below), so
// that ragged batches are balanced; a batch of equal lengths yields exactly one item per workgroup.
//
// plan[0] item counter, plan[1] number of items, plan[2] steps per item (target), plan[3] = 1 when there
// is at most one item per workgroup (then workgroup b takes item b),
// plan[4 + s], s = 0 .. n_seq: items before sequence s.  Sequence s has c_s items per (KV head, row
// group), (KV head, row group) pairs in order, the steps of a pair divided evenly over its c_s items.
constexpr int kPlanHeader = 4;
constexpr int kDecodeWorkgroups = 256;   // one per compute unit
constexpr int kItemOversubscription = 8; // items per workgroup when one item each cannot balance the batch

__device__ __forceinline__ int steps_of(int len, int max_len, int tiles_per_step) {
    const int l = min(max(len, 0), max_len);
    const int tiles = (l + kWave - 1) / kWave;
    return (tiles + tiles_per_step - 1) / tiles_per_step;
}

// Executed by one wavefront (block 0 of the query rotation kernel, which precedes the split-K kernel on
// the stream).
__device__ __forceinline__ void build_plan(const DecodeShape &shp, const int32_t *seq_lens, int tiles_per_step,
                                           int32_t *plan, int lane) {
    const int G = shp.n_kv_heads * shp.n_row_groups;
    // With at most 64 sequences every lane reads its sequence's length once (the three passes below would
    // otherwise each wait for memory again: this kernel is on the critical path of a decode call).
    const bool one_round = shp.n_seq <= kWave;
    const int own_steps = one_round && lane < shp.n_seq ? steps_of(seq_lens[lane], shp.max_len, tiles_per_step) : 0;
    auto steps_at = [&](int s0) {
        if (one_round) return own_steps;
        const int s = s0 + lane;
        return s < shp.n_seq ? steps_of(seq_lens[s], shp.max_len, tiles_per_step) : 0;
    };
    long long total = 0;
    for (int s0 = 0; s0 < shp.n_seq; s0 += kWave) total += steps_at(s0);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) total += __shfl_xor(total, o, kWave);
    total *= G;
    auto count_items = [&](int item) {
        long long cnt = 0;
        for (int s0 = 0; s0 < shp.n_seq; s0 += kWave) cnt += static_cast<long long>((steps_at(s0) + item - 1) / item) * G;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
        return cnt;
    };
    int item = static_cast<int>(max(1LL, (total + kDecodeWorkgroups - 1) / kDecodeWorkgroups));
    if (count_items(item) > kDecodeWorkgroups)
        item = static_cast<int>(max(1LL, (total + kDecodeWorkgroups * kItemOversubscription - 1) /
                                             (kDecodeWorkgroups * kItemOversubscription)));
    int running = 0;
    for (int s0 = 0; s0 < shp.n_seq; s0 += kWave) {
        const int s = s0 + lane;
        const int st = steps_at(s0);
        const int mine = ((st + item - 1) / item) * G;
        int incl = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int other = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += other;
        }
        if (s < shp.n_seq) plan[kPlanHeader + s] = running + incl - mine;
        running += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) {
        plan[kPlanHeader + shp.n_seq] = running;
        plan[0] = 0;
        plan[1] = running;
        plan[2] = item;
        plan[3] = running <= kDecodeWorkgroups ? 1 : 0;
    }
}

struct WaveWork {
    int seq, kvh, grp;
    int64_t pair, group_id;
    int step_begin, step_end, step_stride, step_last, len, n_tiles;
};

// Item `it` (wave-uniform) -> the wavefront's work.
__device__ __forceinline__ void item_work(const DecodeShape &shp, const int32_t *plan, const int32_t *seq_lens, int it,
                                          int wave, int tiles_per_step, WaveWork *ww) {
    const int32_t *before = plan + kPlanHeader;
    int lo, b_lo, b_next, len_lo;        // lo: largest s with before[s] <= it (before[n_seq] > it)
    if (shp.n_seq < kWave) {
        // one round of loads instead of a chain of dependent ones: lane l holds before[l] and the length of
        // sequence l; the lanes whose entry is <= it are counted
        const int l = static_cast<int>(threadIdx.x) & (kWave - 1);
        const int mine = l <= shp.n_seq ? before[l] : 0x7fffffff;
        const int my_len = l < shp.n_seq ? seq_lens[l] : 0;
        const uint64_t le = __ballot(l < shp.n_seq && mine <= it);
        lo = max(__popcll(le) - 1, 0);
        b_lo = __shfl(mine, lo, kWave);
        b_next = __shfl(mine, lo + 1, kWave);
        len_lo = __shfl(my_len, lo, kWave);
        lo = __builtin_amdgcn_readfirstlane(lo);
        b_lo = __builtin_amdgcn_readfirstlane(b_lo);
        b_next = __builtin_amdgcn_readfirstlane(b_next);
        len_lo = __builtin_amdgcn_readfirstlane(len_lo);
    } else {
        int hi = shp.n_seq;
        lo = 0;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (before[mid] <= it) lo = mid; else hi = mid;
        }
        b_lo = before[lo];
        b_next = before[lo + 1];
        len_lo = seq_lens[lo];
    }
    const int G = shp.n_kv_heads * shp.n_row_groups;
    const int c_s = (b_next - b_lo) / G;   // > 0, or `it` would not fall here
    const int local = it - b_lo;
    const int gis = local / c_s, chunk = local % c_s;
    ww->seq = lo;
    ww->group_id = static_cast<int64_t>(lo) * G + gis;
    ww->grp = gis % shp.n_row_groups;
    ww->kvh = gis / shp.n_row_groups;
    ww->pair = static_cast<int64_t>(lo) * shp.n_kv_heads + ww->kvh;
    ww->len = min(max(len_lo, 0), shp.max_len);
    ww->n_tiles = (ww->len + kWave - 1) / kWave;
    const int n_steps = (ww->n_tiles + tiles_per_step - 1) / tiles_per_step;
    const int base = n_steps / c_s, rem = n_steps % c_s;
    const int wb = chunk * base + min(chunk, rem);
    ww->step_end = wb + base + (chunk < rem ? 1 : 0);
    ww->step_begin = wb + wave;
    ww->step_stride = shp.item_waves;
    ww->step_last = ww->step_begin + (ww->step_begin < ww->step_end
                                          ? (ww->step_end - 1 - ww->step_begin) / ww->step_stride
                                          : 0) * ww->step_stride;
}

// Takes the next item for the whole workgroup; false when none is left.  `taken` counts the calls of
// this workgroup.  With at most one item per workgroup (plan[3] = 1: every batch of equal lengths)
// workgroup b simply takes item b, without touching the counter.
__device__ __forceinline__ bool next_item(int32_t *plan, int *slot, int tid, int *taken, int *it) {
    const int n_items = plan[1];
    if (plan[3] != 0) {
        *it = static_cast<int>(blockIdx.x);
        return (*taken)++ == 0 && *it < n_items;
    }
    ++*taken;
    if (tid == 0) *slot = atomicAdd(&plan[0], 1);
    __syncthreads();
    *it = __builtin_amdgcn_readfirstlane(*slot);
    __syncthreads();
    return *it < n_items;
}

// Tiles per step of the split-K kernels: up to d = 128 a lane carries two keys (see the kernel).  The host's
// DecodeShape carries the same number (tiles_per_step) for the kernel that cuts the items.
template <int D>
constexpr int decode_keys_per_lane() { return D <= 128 ? 2 : 1; }

// ---- D0: q_rot = scale * H (s . q), one wavefront per query row ------------------------------
// Output layout per (sequence, KV head, row group): [QS coordinates][RG rows], so that the RG
// values a key needs for one coordinate are adjacent.  Rows past rows_per_kv and coordinates
// past d are written as zeros.
template <int D, int QS>
__global__ __launch_bounds__(kWave) void rotate_queries_kernel(const void *__restrict__ q, int q_is_bf16,
                                                                const uint8_t *__restrict__ signs, DecodeShape s,
                                                                float scale, float *__restrict__ q_rot,
                                                                const int32_t *__restrict__ seq_lens,
                                                                int32_t *__restrict__ plan,
                                                                const uint8_t *__restrict__ signs2,
                                                                float *__restrict__ q2) {
    constexpr int EPL = D / kWave;  // elements per lane (1, 2, 4)
    const int lane = threadIdx.x;
    // block 0 also cuts the work items of the split-K kernel that follows (not used by the many-row kernel)
    if (blockIdx.x == 0 && plan != nullptr) build_plan(s, seq_lens, s.tiles_per_step, plan, lane);
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

    // Optional 1-bit QJL residual (Sec. 3.6): q2 = sqrt(pi / (2 d)) * H diag(s') q_rot per row, [row][d]
    if (q2 != nullptr) {
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int e = lane * EPL + j;
            const bool neg = (signs2[kvh * (D / 8) + (e >> 3)] >> (e & 7)) & 1;
            x[j] = neg ? -x[j] : x[j];
        }
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
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) {
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const float other = __shfl_xor(x[j], m, kWave);
                x[j] = (lane & m) ? other - x[j] : x[j] + other;
            }
        }
        // 1 / sqrt(d) of the Hadamard matrix times sqrt(pi / (2 d)) of the estimator = sqrt(pi / 2) / d
        const float c = 1.2533141373155003f / static_cast<float>(D);
#pragma unroll
        for (int j = 0; j < EPL; ++j) q2[gid * D + lane * EPL + j] = x[j] * c;
    }
}

template <int REP>
__device__ __forceinline__ uint32_t lane_part(int lane) { return (static_cast<uint32_t>(lane) & (REP - 1)) << 4; }

// Chunks of the score pass: 8 / RG triplets each.
template <class P, int RG>
constexpr int score_chunks() { return (P::NTRI + 8 / RG - 1) / (8 / RG); }

struct NoChunkHook {
    template <class C>
    __device__ __forceinline__ void operator()(C) const {}
};

// `hook(integral_constant<chunk>)` is called once per chunk, after the requests of the next chunk and before
// the arithmetic of this one: the caller's slot for work that is to be spread evenly over the pass (the
// matrix-core kernel runs the previous step's P.V and requests this step's values there).  LDS reads the
// hook issues are complete at the top of the next chunk.
template <class P, int RG, int KPL, class Hook = NoChunkHook>
__device__ __forceinline__ void tile_scores(const uint32_t (&w)[KPL][P::NWORDS], const float *__restrict__ qg,
                                            const DecodeTables<P> &tb, int lane, float (&s)[KPL][RG],
                                            const Hook &hook = Hook{}) {
    constexpr int CT = 8 / RG;                       // triplets per chunk
    constexpr int NCHUNK = score_chunks<P, RG>();
    constexpr int QC = CT * 3 * RG;                  // query floats per chunk
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int r = 0; r < RG; ++r) s[k][r] = 0.0f;
    float rgv[KPL][4];                               // the norm centroids of the group last looked up
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) rgv[k][e] = 0.0f;
    float qv[2][QC];
    float4 nv[2][CT][KPL];
    float rv[2][CT][KPL];

    auto request = [&](auto cc) __attribute__((always_inline)) {
        constexpr int ci = decltype(cc)::value;
        constexpr int c0 = ci * CT;
        constexpr int cn = (P::NTRI - c0) < CT ? (P::NTRI - c0) : CT;
        constexpr int buf = ci & 1;
#pragma unroll
        for (int e = 0; e < cn * 3 * RG; ++e) qv[buf][e] = qg[c0 * 3 * RG + e];
        static_for<0, cn>([&](auto tt) {
            constexpr int t = decltype(tt)::value;
            constexpr int i = c0 + t;
            constexpr int c = P::cls(i);
            constexpr int ii = c ? i - P::NT0 : i;   // index within the class
            constexpr int bn = P::bnrm(i);
            constexpr int bd = P::bdir(i);
            using RT = RhoTable<bn>;
            using DT = DirTable<bd>;
            static_for<0, KPL>([&](auto kk) {
                constexpr int k = decltype(kk)::value;
                const uint32_t code = field<P::dir_bit(i), 2 * bd>(w[k]);
                if constexpr (joint_codes(bd, bn)) {
                    using JT = JointTable<bd, bn>;
                    constexpr int nb = P::nrm_bit(i), db = P::dir_bit(i);
                    uint32_t off;
                    if constexpr (JT::BYTE_CODES && (nb & 31) + bn <= 32) {
                        // written out: the compiler's own choice takes four or five instructions
                        const uint32_t dl = __builtin_amdgcn_perm(w[k][db >> 5], lane_part<JT::REP>(lane),
                                                                  0x0c0c0000u | ((4u + ((db & 31) >> 3)) << 8));
                        uint32_t nrm;
                        asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(nrm) : "v"(w[k][nb >> 5]), "n"(nb & 31), "n"(bn));
                        asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(off) : "v"(nrm), "n"(JT::NS), "v"(dl));
                    } else {
                        off = (code << JT::CS) | (field<nb, bn>(w[k]) << JT::NS) | lane_part<JT::REP>(lane);
                    }
                    nv[buf][t][k] = *reinterpret_cast<const float4 *>(
                        reinterpret_cast<const char *>(c ? tb.dir1 : tb.dir0) + off);
                    rv[buf][t][k] = 1.0f;
                } else {
                    if constexpr (ii % RT::NTG == 0) {
                        constexpr int gbit = (c ? P::NRM1_BIT : P::NRM0_BIT) + ii * bn;
                        // the streams are padded to whole bytes, a whole number of groups; the last group
                        // may reach past the class's triplets, never past its stream
                        const uint32_t gi = field_clamped<gbit, RT::BITS, P::NWORDS>(w[k]);
                        const float *entry =
                            (c ? tb.rho1 : tb.rho0) + (gi * RT::REP + (lane & (RT::REP - 1))) * RT::NTG;
                        if constexpr (RT::NTG == 4) {
                            const float4 e = *reinterpret_cast<const float4 *>(entry);
                            rgv[k][0] = e.x; rgv[k][1] = e.y; rgv[k][2] = e.z; rgv[k][3] = e.w;
                        } else if constexpr (RT::NTG == 1) {
                            rgv[k][0] = entry[0];
                        } else {
                            const float2 e = *reinterpret_cast<const float2 *>(entry);
                            rgv[k][0] = e.x; rgv[k][1] = e.y;
                        }
                    }
                    nv[buf][t][k] = (c ? tb.dir1 : tb.dir0)[code * DT::REP + (lane & (DT::REP - 1))];
                    rv[buf][t][k] = rgv[k][ii % RT::NTG];
                }
            });
        });
    };

    request(std::integral_constant<int, 0>{});
    static_for<0, NCHUNK>([&](auto cc) {
        constexpr int ci = decltype(cc)::value;
        constexpr int c0 = ci * CT;
        constexpr int cn = (P::NTRI - c0) < CT ? (P::NTRI - c0) : CT;
        constexpr int buf = ci & 1;
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): the inputs of this chunk have arrived
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (ci + 1 < NCHUNK) request(std::integral_constant<int, ci + 1>{});
        hook(cc);
        static_for<0, cn>([&](auto tt) {
            constexpr int t = decltype(tt)::value;
            static_for<0, KPL>([&](auto kk) {
                constexpr int k = decltype(kk)::value;
                const float4 n = nv[buf][t][k];
                float tx = n.x, ty = n.y, tz = n.z;
                if constexpr (!joint_codes(P::bdir(c0 + t), P::bnrm(c0 + t))) {
                    const float rho = rv[buf][t][k];
                    tx *= rho; ty *= rho; tz *= rho;
                }
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    s[k][r] = fmaf(qv[buf][(3 * t) * RG + r], tx, s[k][r]);
                    s[k][r] = fmaf(qv[buf][(3 * t + 1) * RG + r], ty, s[k][r]);
                    s[k][r] = fmaf(qv[buf][(3 * t + 2) * RG + r], tz, s[k][r]);  // rotated queries are zero past d
                }
            });
        });
        // The accumulators pass through an empty volatile asm at the end of each chunk: instruction
        // selection orders side-effect-free arithmetic freely within the block, and without this anchor it
        // may defer every multiply-add past the last chunk, keeping the whole query live (spilled).
#pragma unroll
        for (int k = 0; k < KPL; ++k)
#pragma unroll
            for (int r = 0; r < RG; ++r) asm volatile("" : "+v"(s[k][r]));
        __builtin_amdgcn_sched_barrier(0);
    });
}

// Byte offset, in the joint table of its class, of the entry of triplet I of the record `w` for this lane.
template <class P, int I>
__device__ __forceinline__ uint32_t joint_offset(const uint32_t (&w)[P::NWORDS], int lane) {
    constexpr int bn = P::bnrm(I), bd = P::bdir(I);
    using JT = JointTable<bd, bn>;
    constexpr int nb = P::nrm_bit(I), db = P::dir_bit(I);
    if constexpr (JT::BYTE_CODES && (nb & 31) + bn <= 32) {
        const uint32_t dl = __builtin_amdgcn_perm(w[db >> 5], lane_part<JT::REP>(lane),
                                                  0x0c0c0000u | ((4u + ((db & 31) >> 3)) << 8));
        uint32_t nrm, off;
        asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(nrm) : "v"(w[nb >> 5]), "n"(nb & 31), "n"(bn));
        asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(off) : "v"(nrm), "n"(JT::NS), "v"(dl));
        return off;
    } else {
        return (field<db, 2 * bd>(w) << JT::CS) | (field<nb, bn>(w) << JT::NS) | lane_part<JT::REP>(lane);
    }
}

// ---- D2-D4 on the matrix cores ------------------------------------------------------------------------
// Once the table entry of a triplet is in hand, its contribution to the scores of RG query rows is a dense
// 4 x 4 x 4 product per group of four keys: rows x (x, y, z, 0) times (x, y, z, 0) x keys.
// v_mfma_f32_4x4x4_16b_bf16 multiplies 16 such blocks at once: lane l supplies row l % 4 of A and column
// l % 4 of B of block l / 4 (four bf16 each) and receives column l % 4 of D, register v = row v.  With
// A = the rotated queries (row l % 4; the same in every block) and B = the table entry of lane l's own key,
// lane l ends up with the scores of ITS key for four query rows: the layout the softmax below expects, with
// no cross-lane traffic.  fp32 accuracy comes from bf16 pairs: q = q_hi + q_lo, entry = e_hi + e_lo, and
// three products per triplet (hi hi, lo hi, hi lo; the dropped lo lo term is below 2^-16 of the product),
// accumulated in fp32 by the instruction.
//
// Query operands of a work item, staged in LDS by the workgroup: entry (triplet i, row r) = split_triplet of
// (q_rot[r][3 i], q_rot[r][3 i + 1], q_rot[r][3 i + 2]); rows are padded to a multiple of four with zeros.
template <class P, int RG>
struct QueryOperands {
    static constexpr int ROWS = RG <= 4 ? 4 : 8;
    uint4 e[P::NTRI][ROWS];
};

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float mx_f32x4_t __attribute__((ext_vector_type(4)));

// All operands come from LDS (no scalar loads in the pass), so the hardware counter of outstanding LDS reads
// is exact and the reads of a triplet can be issued LA triplets before its products.  `hook` as in
// tile_scores, called every 8 / RG triplets.
// LOOKAHEAD: triplets requested ahead of their products (4 hides the LDS latency for a wavefront that has its
// SIMD to itself; a kernel with two wavefronts per SIMD and registers to spare for neither asks for less).
template <class P, int RG, int KPL, class Hook = NoChunkHook, int LOOKAHEAD = 4>
__device__ __forceinline__ void tile_scores_mx(const uint32_t (&w)[KPL][P::NWORDS], const QueryOperands<P, RG> &qop,
                                               const DecodeTables<P> &tb, int lane, float (&s)[KPL][RG],
                                               const Hook &hook = Hook{}) {
    constexpr int CT = 8 / RG;
    constexpr int NSET = QueryOperands<P, RG>::ROWS / 4;
    constexpr int LA = P::NTRI < LOOKAHEAD ? P::NTRI : LOOKAHEAD;   // triplets requested ahead
    constexpr int NB = LA + 1;
    uint4 ev[NB][KPL], qv[NB][NSET];
    mx_f32x4_t d_main[KPL][NSET], d_cross[KPL][NSET];
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int h = 0; h < NSET; ++h) {
            d_main[k][h] = mx_f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
            d_cross[k][h] = mx_f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
        }
    const char *q_lane = reinterpret_cast<const char *>(&qop.e[0][0]) + (lane & 3) * 16;
    auto request = [&](auto ii) __attribute__((always_inline)) {
        constexpr int i = decltype(ii)::value;
        constexpr int slot = i % NB;
        constexpr int c = P::cls(i);
#pragma unroll
        for (int k = 0; k < KPL; ++k)
            ev[slot][k] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(c ? tb.dir1 : tb.dir0) +
                                                           joint_offset<P, i>(w[k], lane));
#pragma unroll
        for (int h = 0; h < NSET; ++h)
            qv[slot][h] = *reinterpret_cast<const uint4 *>(q_lane + (i * QueryOperands<P, RG>::ROWS + 4 * h) * 16);
    };
    static_for<0, LA>(request);
    static_for<0, P::NTRI>([&](auto ii) {
        constexpr int i = decltype(ii)::value;
        constexpr int slot = i % NB;
        if constexpr (i + LA < P::NTRI) request(std::integral_constant<int, i + LA>{});
        if constexpr (i % CT == 0) hook(std::integral_constant<int, i / CT>{});
#pragma unroll
        for (int h = 0; h < NSET; ++h) {
            union { uint32_t u[2]; s16x4_t v; } q_hi, q_lo;
            q_hi.u[0] = qv[slot][h].x; q_hi.u[1] = qv[slot][h].y;
            q_lo.u[0] = qv[slot][h].z; q_lo.u[1] = qv[slot][h].w;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                union { uint32_t u[2]; s16x4_t v; } e_hi, e_lo;
                e_hi.u[0] = ev[slot][k].x; e_hi.u[1] = ev[slot][k].y;
                e_lo.u[0] = ev[slot][k].z; e_lo.u[1] = ev[slot][k].w;
                d_main[k][h] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(q_hi.v, e_hi.v, d_main[k][h], 0, 0, 0);
                d_cross[k][h] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(q_lo.v, e_hi.v, d_cross[k][h], 0, 0, 0);
                d_cross[k][h] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(q_hi.v, e_lo.v, d_cross[k][h], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int r = 0; r < RG; ++r) s[k][r] = d_main[k][r / 4][r % 4] + d_cross[k][r / 4][r % 4];
}

template <int RG>
__device__ __forceinline__ void store_scores(const DecodeShape &shp, const WaveWork &ww, float *scores_out, int tok,
                                             const float (&s)[RG]) {
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const int row = ww.grp * RG + r;
        if (row < shp.rows_per_kv) {
            const int qi = row / shp.heads_per_kv, head = ww.kvh * shp.heads_per_kv + row % shp.heads_per_kv;
            scores_out[((static_cast<int64_t>(ww.seq) * shp.n_q + qi) * shp.n_q_heads + head) * shp.t_capacity + tok] =
                s[r];
        }
    }
}

// ---- bf16 values: P.V on the matrix cores -------------------------------------------------------
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] B[32x16]; lane l holds row l%16 of A and
// column l%16 of B, each for the 8 k-slots of lane group l/16, and rows 4*(l/16)..+3 of column l%16
// of D.  Here M = probability rows, K = keys, N = channels:
//   * a 64-key tile is two k-steps; k-slot (g, j) of step ks is key 32*ks + 4*j + g, so that one
//     wave-wide value load (fixed j) reads 4 consecutive value rows (measured faster than 4 rows that
//     lie 8 apart);
//   * lane (n, g) loads CPL = d/16 channels of its 8 keys per k-step, 16 bytes (8 bytes at d = 64) of every
//     256-byte piece of the row, so that one load instruction of the wavefront reads whole cache lines;
//     N-block c of the MFMA is the channel set {lane n's c-th channel}, so B operands are byte permutes of
//     the loaded registers and values are never converted;
//   * values come through buffer loads whose descriptor ends at the sequence's last token: rows past
//     it read as zeros without any address clamping;
//   * a probability is split into two bf16 numbers, hi = its upper 16 bits and lo = the rest, which
//     occupy rows r and RP + r of A; the two partial results are added at the end.  The relative
//     error of hi + lo is below 2^-16.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Keys per lane and step of the bf16-value kernel.  The kernel runs one wavefront per SIMD (all 512
// vector registers of a lane): measured faster than two wavefronts with half the registers each,
// because a step's values (16 KB per 64 keys at d = 128) stay in flight in registers during the whole
// score phase without spilling.  Up to d = 128 a lane carries two keys, so that every scalar query
// chunk, every wave-wide maximum and every accumulator rescale serves 128 keys.
template <int KPL>
constexpr int prob_row() { return KPL * kWave + 8; }  // bf16 per probability row in LDS: keys + 8 pad

template <class P, int KPL>
struct DecodeSmemMfma {
    DecodeTables<P> tb;
    uint16_t pbuf[kDecodeWaves][16][prob_row<KPL>()];
};

// Optional 1-bit QJL residual (Sec. 3.6).  The correction of a key, sum_j sigma_j q2_j per query row, is
// looked up a byte of sign bits at a time: entry [position][byte value][row] holds the signed sum of the 8
// q2 coordinates of that byte.  The table is rebuilt per work item (it depends on the queries).
template <class P, int RG>
constexpr int qjl_table_floats() { return (P::D / 8) * 256 * RG; }
template <class P, int RG>
constexpr bool qjl_fits() {
    return sizeof(DecodeSmemMfma<P, decode_keys_per_lane<P::D>()>) + qjl_table_floats<P, RG>() * 4 +
               sizeof(QueryOperands<P, RG>) + 64 <= 160 * 1024;
}

// SCORES: also store the scaled scores (a second instantiation, so that the usual one carries none of
// the addressing state of that store through its loop).
// QJL: add the 1-bit QJL residual correction of Sec. 3.6 to every score (side-car `qjl`, second rotated
// queries `q2`).
// PAGED: `cache` and `v` are pools of 64-token pages, [page][KV head] tiles each (a key tile in the device
// layout of the contiguous cache, a value tile of 64 rows), and logical tile j of sequence s lives in page
// pt_table[s * pt_stride + j] (ids outside [0, pt_pages) are clamped: a bad table reads wrong pages, never
// outside the pools).  The page ids of a step are read one step before its loads are issued.
template <class P, int RG, bool SCORES, bool QJL, bool PAGED = false>
__global__ __launch_bounds__(kDecodeWaves *kWave) __attribute__((amdgpu_waves_per_eu(1, 1))) void decode_kernel_mfma(
    DeviceBooks books, DecodeShape shp, const float *__restrict__ q_rot, const uint4 *__restrict__ cache,
    const uint32_t *__restrict__ v, const int32_t *__restrict__ seq_lens, float *__restrict__ part_ml,
    float *__restrict__ part_acc, float *__restrict__ scores_out, int32_t *__restrict__ plan,
    const unsigned char *__restrict__ qjl, const float *__restrict__ q2, const int32_t *__restrict__ pt_table,
    int32_t pt_stride, int32_t pt_pages) {
    // (the table as a restrict-qualified kernel argument of its own: its loads are then known not to be
    // clobbered by the kernel's stores and become scalar loads)
    constexpr int D = P::D;
    constexpr int KPL = decode_keys_per_lane<D>();
    constexpr bool AHEAD = D <= 128;       // P.V runs one step behind the scores, inside the next score pass
    constexpr int KS = 2 * KPL;            // k-steps of 32 keys per step
    constexpr int CPL = D / 16;            // channels per lane chunk = N-blocks
    constexpr int CW = CPL / 2;            // 32-bit words per chunk
    constexpr int RP = RG < 4 ? 4 : RG;    // probability rows padded to a multiple of 4
    constexpr int ROWB = D * 2;            // bytes per value row
    constexpr int TILEB = P::GRANULES * kWave * 16;  // bytes per cache tile
    constexpr int PROW = prob_row<KPL>();
    constexpr int QW = D / 32;             // sign words per key of the QJL side-car
    constexpr int TQ = kWave * (D / 8 + 2);  // side-car bytes per tile
    // static, so that table addresses are compile-time constants that fold into the LDS instructions
    constexpr bool MX = mx_scores<P>();    // scores on the matrix cores (every plan up to 3 bits per coordinate)
    __shared__ DecodeSmemMfma<P, KPL> sm;
    __shared__ __attribute__((aligned(16))) float qtab[QJL ? qjl_table_floats<P, RG>() : 4];
    __shared__ __attribute__((aligned(16))) uint4 qop_store[MX ? P::NTRI * QueryOperands<P, RG>::ROWS : 1];
    const QueryOperands<P, RG> &qop = *reinterpret_cast<const QueryOperands<P, RG> *>(&qop_store[0]);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
    for (int e = tid; e < kDecodeWaves * 16 * PROW; e += kDecodeWaves * kWave) (&sm.pbuf[0][0][0])[e] = 0;
    // The tables are built inside the item loop, after the first item's first loads have been issued:
    // those do not depend on the tables, and their latency covers the build.
    bool tables_built = false;

    __shared__ int item_slot;
    // per item (set in the item loop below; the helpers capture them by reference)
    WaveWork ww;
    const float *qg = q_rot;
    const char *k_region = reinterpret_cast<const char *>(cache);
    const char *v_pair = reinterpret_cast<const char *>(v);
    const int n16 = lane & 15, g4 = lane >> 4;
    const uint32_t k_lane = lane * 16u;
    // A value row is read in pieces of 16 lanes x LANEB bytes, each piece contiguous (whole cache lines per
    // load instruction: with the non-temporal hint a line touched by two instructions may be fetched twice).
    // Lane n16 holds bytes [n16 LANEB, (n16 + 1) LANEB) of every piece: at d = 256 its 16 channels are
    // 8 n16 .. + 7 and 128 + 8 n16 .. + 7, and N-block c of the P.V product is channel
    // (c / 8) 128 + 8 n16 + c % 8.
    constexpr int LANEB = CPL * 2 < 16 ? CPL * 2 : 16;
    // Byte offsets of this lane's channels in its rows 32 ks + 4 j + g4: one register per JB values of j,
    // the others reached by immediate offsets (below 4096).
    constexpr int JB = 4096 / (4 * ROWB) < 8 ? 4096 / (4 * ROWB) : 8;
    int v_lane[KS][8 / JB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int h = 0; h < 8 / JB; ++h) v_lane[ks][h] = (32 * ks + 4 * JB * h + g4) * ROWB + n16 * LANEB;
    const int ppos = (lane & 32) + 8 * (lane & 3) + ((lane & 31) >> 2);  // slot of key `lane` in a pbuf row

    // Only the words that hold record bytes are loaded: a register written by a load but never read
    // may be reused at once by the compiler, which then has to wait for that load first.
    auto load_record = [&](int64_t tile, uint32_t (&w)[P::NWORDS]) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));
        constexpr int USED = (P::RECORD_BYTES + 3) / 4;
        const char *src = k_region + tile * TILEB;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            const char *gp = src + g * (kWave * 16) + k_lane;
            constexpr int kFull = 4;
            const int n = (USED - 4 * g) < kFull ? (USED - 4 * g) : kFull;
            // (global address space said explicitly: the laundered base pointer below would otherwise make these
            // flat loads, which count against the LDS / scalar wait counter as well)
            typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
            typedef const u32x4_t __attribute__((address_space(1))) *g4_t;
            typedef const u32x3_t __attribute__((address_space(1))) *g3_t;
            typedef const u32x2_t __attribute__((address_space(1))) *g2_t;
            typedef const uint32_t __attribute__((address_space(1))) *g1_t;
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
    // The records of a step; a tile past the sequence's last one is replaced by the last one (its keys
    // are masked out by position), so that nothing outside the tiles that hold tokens is read.
    auto load_records = [&](int step, uint32_t (&w)[KPL][P::NWORDS]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) load_record(min(step * KPL + k, ww.n_tiles - 1), w[k]);
    };
    // PAGED: the page ids of the tiles of a step (the last tile's for tiles past it) are read as they are, one
    // step ahead; the position in the pools (in tiles) is computed from them when the step's loads are issued,
    // so that nothing waits for the table right after asking it.
    // The ids come through the vector memory path (every lane reads the same entry), asked for before the
    // step's other loads: the wait for them one step later then covers only loads that are long complete.  As
    // scalar loads they shared a counter with the query chunks, whose first wait of a step also waited for a
    // table entry that had missed the scalar cache.
    int lane_zero = 0;
    if constexpr (PAGED) asm volatile("" : "+v"(lane_zero));
    auto page_ids = [&](int step, int (&page)[KPL]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int tile = max(min(step * KPL + k, ww.n_tiles - 1), 0);
            page[k] = pt_table[static_cast<int64_t>(ww.seq) * pt_stride + tile + lane_zero];
        }
    };
    auto page_slots = [&](const int (&page)[KPL], int64_t (&slot)[KPL]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int id = __builtin_amdgcn_readfirstlane(page[k]);
            slot[k] = static_cast<int64_t>(min(max(id, 0), pt_pages - 1)) * shp.n_kv_heads + ww.kvh;
        }
    };
    auto load_records_at = [&](const int64_t (&slot)[KPL], uint32_t (&w)[KPL][P::NWORDS]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) load_record(slot[k], w[k]);
    };
    int64_t slot_cur[KPL];   // PAGED: pool positions of the step being worked on
    int page_nxt[KPL];       // PAGED: page ids of the wave's next step
    // QJL side-car of a step: per key d / 32 words of sign bits (bit set: negative) and the fp16 residual
    // norm; tile layout [word][key] then [key].
    const char *j_region = reinterpret_cast<const char *>(qjl);
    auto load_sidecar = [&](int step, uint32_t (&sc)[KPL][QW + 1]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const char *src = j_region + static_cast<int64_t>(min(step * KPL + k, ww.n_tiles - 1)) * TQ;
#pragma unroll
            for (int wq = 0; wq < QW; ++wq)
                sc[k][wq] = *reinterpret_cast<const uint32_t *>(src + wq * (kWave * 4) + lane * 4);
            sc[k][QW] = *reinterpret_cast<const uint16_t *>(src + QW * (kWave * 4) + lane * 2);
        }
    };
    // PAGED: the side-car is a pool of [page][KV head] tiles like the keys'; slot = page * n_kv_heads + KV head
    auto load_sidecar_at = [&](const int64_t (&slot)[KPL], uint32_t (&sc)[KPL][QW + 1]) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const char *src = j_region + slot[k] * TQ;
#pragma unroll
            for (int wq = 0; wq < QW; ++wq)
                sc[k][wq] = *reinterpret_cast<const uint32_t *>(src + wq * (kWave * 4) + lane * 4);
            sc[k][QW] = *reinterpret_cast<const uint16_t *>(src + QW * (kWave * 4) + lane * 2);
        }
    };
    // Sum over the d / 8 sign bytes of a key of the table rows they select: q2 . sigma per query row.
    auto qjl_dot = [&](const uint32_t (&sc)[QW + 1], float (&corr)[RG]) {
#pragma unroll
        for (int r = 0; r < RG; ++r) corr[r] = 0.0f;
#pragma unroll
        for (int wq = 0; wq < QW; ++wq)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t byte = (sc[wq] >> (8 * b)) & 0xffu;
                const float *row = &qtab[((4 * wq + b) * 256 + byte) * RG];
                if constexpr (RG == 1) {
                    corr[0] += row[0];
                } else if constexpr (RG == 2) {
                    const float2 t = *reinterpret_cast<const float2 *>(row);
                    corr[0] += t.x; corr[1] += t.y;
                } else {
#pragma unroll
                    for (int h = 0; h < RG / 4; ++h) {
                        const float4 t = *reinterpret_cast<const float4 *>(row + 4 * h);
                        corr[4 * h] += t.x; corr[4 * h + 1] += t.y; corr[4 * h + 2] += t.z; corr[4 * h + 3] += t.w;
                    }
                }
            }
    };
    float m_run[RG], l_lane[RG];
    f32x4_t acc[CPL];

    // Values come through a buffer descriptor that covers a step's rows up to the sequence's last token
    // (rows past it read as zero; their probabilities are zero too); the descriptor of a step that does
    // not exist is empty, its loads move nothing.
    auto values_of = [&](int step, bool exists) {
        const int t0 = step * (KPL * kWave);
        const int n_valid = exists ? min(KPL * kWave, ww.len - t0) : 0;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(v_pair + static_cast<int64_t>(t0) * ROWB), 0,
                                                 n_valid * ROWB, 0x00020000);
    };
    // PAGED: tile k of a step has a descriptor of its own.  The lanes address rows relative to the step's
    // first row, so the descriptor starts 64 k rows before the tile (nothing below the tile is addressed
    // through it) and ends with the tile's last token.
    auto values_at = [&](int step, int k, int64_t slot, bool exists) {
        // (wave-uniform by construction; said so explicitly, or the descriptor may end up in vector registers
        // and every load through it in a loop over its distinct values)
        const int n_valid =
            __builtin_amdgcn_readfirstlane(exists ? min(max(ww.len - (step * KPL + k) * kWave, 0), kWave) : 0);
        const int64_t off = (slot - k) * (kWave * ROWB);
        const uint32_t off_lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(off));
        const uint32_t off_hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(off) >> 32));
        const char *base = v_pair + static_cast<int64_t>((static_cast<uint64_t>(off_hi) << 32) | off_lo);
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0,
                                                 n_valid > 0 ? (k * kWave + n_valid) * ROWB : 0, 0x00020000);
    };
    // Values and records are read once and never again: the loads carry the non-temporal hint (bit 1 of the
    // buffer intrinsic's cache policy, the nt bit of a global load), which keeps the stream from displacing
    // what the caches hold.  Measured on the Llama-shaped batch: 0.243 -> 0.205 ms for the whole kernel.
    // this lane's part of k-step ks: 8 rows x CPL channels
    auto load_values = [&](__amdgpu_buffer_rsrc_t rsrc, int ks, uint32_t (&vk)[8][CW]) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (CW == 2) {
                const u32x2_t x =
                    __builtin_amdgcn_raw_buffer_load_b64(rsrc, v_lane[ks][j / JB] + (j % JB) * (4 * ROWB), 0, kStreamPolicy);
                vk[j][0] = x.x; vk[j][1] = x.y;
            } else {
#pragma unroll
                for (int q4 = 0; q4 < CW / 4; ++q4) {
                    const u32x4_t x = __builtin_amdgcn_raw_buffer_load_b128(
                        rsrc, v_lane[ks][j / JB] + (j % JB) * (4 * ROWB) + 16 * LANEB * q4, 0, kStreamPolicy);
                    vk[j][4 * q4] = x.x; vk[j][4 * q4 + 1] = x.y; vk[j][4 * q4 + 2] = x.z; vk[j][4 * q4 + 3] = x.w;
                }
            }
        }
    };
    uint32_t vr[KS][8][CW];  // values: of the previous step until its P.V piece has run, then of the current step
    // P.V of one step is cut into KS * CW pieces: piece (ks, q) multiplies the probabilities of k-step ks with
    // the two channel blocks 2 q and 2 q + 1, whose B operands are byte permutes of word q of the k-step's
    // eight value registers.  A piece's A operand (16 bytes of the probability rows in LDS) is read one
    // piece ahead.
    constexpr int NPIECE = KS * CW;
    auto pv_operand = [&](int ks) {
        return *reinterpret_cast<const uint4 *>(&sm.pbuf[wave][n16][32 * ks + 8 * g4]);
    };
    auto pv_piece = [&](auto pp, const uint4 &pa_bits) __attribute__((always_inline)) {
        constexpr int ks = decltype(pp)::value / CW, q = decltype(pp)::value % CW;
        union { uint4 u; bf16x8_t b; } pa;
        pa.u = pa_bits;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            union { uint32_t u[4]; bf16x8_t b; } vb;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                vb.u[jj] = __builtin_amdgcn_perm(vr[ks][2 * jj + 1][q], vr[ks][2 * jj][q], h ? 0x07060302u : 0x05040100u);
            acc[2 * q + h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.b, vb.b, acc[2 * q + h], 0, 0, 0);
        }
    };
    // One step.  Up to d = 128 the step is software pipelined with P.V one step behind the scores: the score
    // pass of step n carries, spread over its chunks, the P.V pieces of step n - 1 (whose probabilities sit in
    // LDS since the end of that step) and, as soon as the last piece of a k-step has read its value registers,
    // the loads of step n's own values into them.  Matrix-core work thus overlaps the vector arithmetic of the
    // scores, and -- what matters more with a single in-order wavefront per SIMD -- the value loads enter the
    // compute unit's memory pipeline a k-step at a time at the pace of the arithmetic, not in one burst per step
    // whose issue stalls the wavefront.  The first step of an item multiplies zeros (the value registers are
    // cleared at the item's start), the last step's P.V runs after the loop.  At d = 256 (registers: holding a
    // step's values across the score pass spills there) the values are requested at the top of the step and
    // P.V follows the softmax.  The records of the wave's next step are requested first thing
    // and are used one call later.  The step loop below is unrolled by two with the two record buffers
    // swapping roles, so that no register copies (and no full memory wait in front of them) carry the
    // prefetched records over.
    auto process_step = [&](int step, const uint32_t (&w)[KPL][P::NWORDS], uint32_t (&w_next)[KPL][P::NWORDS],
                            const uint32_t (&sc)[KPL][QW + 1], uint32_t (&sc_next)[KPL][QW + 1])
                            __attribute__((always_inline)) {
        const int t0 = step * (KPL * kWave);
        const int n_valid = min(KPL * kWave, ww.len - t0);
        // always issued (the wave's last step re-reads its own records): a branch here would make the compiler
        // wait for every outstanding load first
        const int step_nx = min(step + ww.step_stride, ww.step_last);
        __amdgpu_buffer_rsrc_t v_cur[KPL];   // this step's values, per tile of the step (all the same unless PAGED)
        int64_t slot_nxt[KPL];
        if constexpr (PAGED) {
            page_slots(page_nxt, slot_nxt);
            page_ids(min(step_nx + ww.step_stride, ww.step_last), page_nxt);   // used one step from here
        }
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            if constexpr (PAGED) v_cur[k] = values_at(step, k, slot_cur[k], true);
            else v_cur[k] = values_of(step, true);
        }
        if constexpr (!AHEAD) {   // d = 256: the registers hold one step's values only while it is worked on
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) load_values(v_cur[ks / 2], ks, vr[ks]);
        }
        if constexpr (PAGED) {
            load_records_at(slot_nxt, w_next);
            if constexpr (QJL) load_sidecar_at(slot_nxt, sc_next);
#pragma unroll
            for (int k = 0; k < KPL; ++k) slot_cur[k] = slot_nxt[k];
        } else {
            load_records(step_nx, w_next);
            if constexpr (QJL) load_sidecar(min(step + ww.step_stride, ww.step_last), sc_next);
        }
        // The loads above feed the NEXT step, which sits behind a branch in the unrolled loop; without this
        // barrier the compiler sinks them into that branch, i.e. to the top of the step that uses them, and
        // every second step waits for a full memory round trip.
        asm volatile("" ::: "memory");
        // D2-D4: scores (queries carry the softmax scale already).  The query offset (always 0) is
        // laundered per step: otherwise the loop-invariant scalar loads of the whole query are hoisted
        // out of the step loop and hundreds of scalar registers spill.
        float s[KPL][RG];
        int q_off = 0;
        asm volatile("" : "+s"(q_off));
        if constexpr (AHEAD) {
            // chunk c runs pieces [c NPIECE / NCH, (c + 1) NPIECE / NCH) and reads the A operands of chunk c + 1's
            constexpr int NCH = score_chunks<P, RG>();
            uint4 pa_bits[NPIECE];
            static_for<0, NPIECE / NCH>([&](auto pp) { pa_bits[decltype(pp)::value] = pv_operand(decltype(pp)::value / CW); });
            auto pv_in_chunk = [&](auto cc) __attribute__((always_inline)) {
                constexpr int ci = decltype(cc)::value;
                constexpr int lo = ci * NPIECE / NCH, hi = (ci + 1) * NPIECE / NCH;
                constexpr int hi_next = ci + 1 < NCH ? (ci + 2) * NPIECE / NCH : hi;
                static_for<hi, hi_next>([&](auto pp) { pa_bits[decltype(pp)::value] = pv_operand(decltype(pp)::value / CW); });
                static_for<lo, hi>([&](auto pp) {
                    constexpr int pi = decltype(pp)::value;
                    pv_piece(pp, pa_bits[pi]);
                    if constexpr (pi % CW == CW - 1) load_values(v_cur[(pi / CW) / 2], pi / CW, vr[pi / CW]);
                });
            };
            if constexpr (MX) tile_scores_mx<P, RG, KPL>(w, qop, sm.tb, lane, s, pv_in_chunk);
            else tile_scores<P, RG, KPL>(w, qg + q_off, sm.tb, lane, s, pv_in_chunk);
            // the probabilities of the previous step have been read: the new ones may overwrite them
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else {
            if constexpr (MX) tile_scores_mx<P, RG, KPL>(w, qop, sm.tb, lane, s);
            else tile_scores<P, RG, KPL>(w, qg + q_off, sm.tb, lane, s);
        }
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const float gamma = __uint_as_float(w[k][0]);
            const bool valid = k * kWave + lane < n_valid;
            if constexpr (QJL) {
                // Sec. 3.6: q . k = gamma (q_rot . u^ + gamma_r q2 . sigma), the estimator's constant is in q2
                float corr[RG];
                qjl_dot(sc[k], corr);
                const float gamma_r = __half2float(__ushort_as_half(static_cast<unsigned short>(sc[k][QW])));
#pragma unroll
                for (int r = 0; r < RG; ++r) s[k][r] = fmaf(gamma_r, corr[r], s[k][r]);
            }
#pragma unroll
            for (int r = 0; r < RG; ++r) s[k][r] = valid ? s[k][r] * gamma : -INFINITY;
            if constexpr (SCORES) {
                // the kernel with the residual is built once; it looks at the pointer
                if (valid && (!QJL || scores_out != nullptr))
                    store_scores<RG>(shp, ww, scores_out, t0 + k * kWave + lane, s[k]);
            }
        }
        // D5: online softmax, one running maximum per row for the whole wave
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
                const float p = exp2_raw((s[k][r] - m_new) * kLog2e);
                psum += p;
                const uint32_t pb = __float_as_uint(p);
                const float lo = p - __uint_as_float(pb & 0xffff0000u);
                sm.pbuf[wave][r][k * kWave + ppos] = static_cast<uint16_t>(pb >> 16);
                sm.pbuf[wave][RP + r][k * kWave + ppos] = static_cast<uint16_t>(__float_as_uint(lo) >> 16);
            }
            l_lane[r] = fmaf(l_lane[r], alpha[r], psum);
        }
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
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if constexpr (!AHEAD) {
            // D6: P.V of this step
            static_for<0, NPIECE>([&](auto pp) { pv_piece(pp, pv_operand(decltype(pp)::value / CW)); });
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    };
    uint32_t w_a[KPL][P::NWORDS], w_b[KPL][P::NWORDS];
    uint32_t sc_a[KPL][QW + 1], sc_b[KPL][QW + 1];
    int it, taken = 0;
    while (next_item(plan, &item_slot, tid, &taken, &it)) {
        item_work(shp, plan, seq_lens, it, wave, KPL, &ww);
        qg = q_rot + ww.group_id * (P::QS * RG);
        if constexpr (QJL) {
            // Every wavefront is past the previous item here (next_item's barriers, or this is the
            // workgroup's only item).  Thread `tid` is the byte value: entry [pos][tid][r] is the sum of
            // the 8 coordinates of q2 at position pos, each negated where tid has its bit set.
            const float *q2g = q2 + ww.group_id * (RG * D);
            for (int pos = 0; pos < D / 8; ++pos)
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    float t = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float x = q2g[r * D + 8 * pos + e];
                        t += ((tid >> e) & 1) ? -x : x;
                    }
                    qtab[(pos * 256 + tid) * RG + r] = t;
                }
            __syncthreads();
            j_region = reinterpret_cast<const char *>(qjl) + (PAGED ? 0 : ww.pair * (shp.t_capacity / kWave) * TQ);
        }
        // Addresses are a wave-uniform base (scalar registers) plus a small per-lane byte offset.
        if constexpr (PAGED) {
            k_region = reinterpret_cast<const char *>(cache);
            v_pair = reinterpret_cast<const char *>(v);
        } else {
            k_region = reinterpret_cast<const char *>(cache) + ww.pair * shp.t_capacity * (P::GRANULES * 16);
            v_pair = reinterpret_cast<const char *>(v) + ww.pair * shp.t_capacity * ROWB;
        }
        // The record pointer loses its "read-only, never aliased" provenance here: loads known to be invariant
        // may be moved across any barrier, and the compiler then sinks the prefetch of the next step's records
        // into the (conditional) step that uses them.
        // (not at d = 256: holding the next step's records through a whole step spills registers there)
        if constexpr (AHEAD) {
            const uint64_t bits = reinterpret_cast<uint64_t>(k_region);
            uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits));
            uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits >> 32));
            asm volatile("" : "+s"(lo), "+s"(hi));
            k_region = reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
        }
#pragma unroll
        for (int r = 0; r < RG; ++r) { m_run[r] = -INFINITY; l_lane[r] = 0.0f; }
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

        if (ww.step_begin < ww.step_end) {
            if constexpr (PAGED) {
                int page_first[KPL];
                page_ids(ww.step_begin, page_first);
                page_ids(min(ww.step_begin + ww.step_stride, ww.step_last), page_nxt);
                page_slots(page_first, slot_cur);
                load_records_at(slot_cur, w_a);
                if constexpr (QJL) load_sidecar_at(slot_cur, sc_a);
            } else {
                load_records(ww.step_begin, w_a);
                if constexpr (QJL) load_sidecar(ww.step_begin, sc_a);
            }
        }
        if constexpr (AHEAD) {
            // The first step's P.V pieces multiply zeros (by whatever probabilities the previous item left in
            // LDS).  The zeros come from loads through an empty descriptor, which move nothing: the wavefront
            // then enters the step loop with the same sequence of outstanding loads as a later iteration has,
            // and the wait counts the compiler derives for the loop are those of the steady state (it takes the
            // stricter of the two ways into the loop).
            const __amdgpu_buffer_rsrc_t v_none = values_of(0, false);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) load_values(v_none, ks, vr[ks]);
        }
        if (!tables_built) {   // workgroup-uniform
            build_tables<P, MX>(sm.tb, books, tid, kDecodeWaves * kWave);
            tables_built = true;
        }
        if constexpr (MX) {
            // The item's rotated queries as matrix-core operands.  Every wavefront is past the previous item
            // here (next_item's barriers, or this is the workgroup's only item).
            constexpr int ROWS = QueryOperands<P, RG>::ROWS;
            uint4 *dst = reinterpret_cast<uint4 *>(&qop_store[0]);
            for (int e = tid; e < P::NTRI * ROWS; e += kDecodeWaves * kWave) {
                const int i = e / ROWS, r = e % ROWS;
                float x = 0.0f, y = 0.0f, z = 0.0f;
                if (r < RG) {   // (the rotated queries are stored [coordinate][row], zero past d)
                    x = qg[(3 * i) * RG + r];
                    y = qg[(3 * i + 1) * RG + r];
                    z = qg[(3 * i + 2) * RG + r];
                }
                dst[e] = split_triplet(x, y, z);
            }
            __syncthreads();
        }
        for (int step = ww.step_begin; step < ww.step_end; step += 2 * ww.step_stride) {
            process_step(step, w_a, w_b, sc_a, sc_b);
            if (step + ww.step_stride < ww.step_end) process_step(step + ww.step_stride, w_b, w_a, sc_b, sc_a);
        }
        if constexpr (AHEAD) {   // D6 of the wave's last step
            static_for<0, NPIECE>([&](auto pp) { pv_piece(pp, pv_operand(decltype(pp)::value / CW)); });
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }

        // D7: add the hi and lo partial results (lane groups RP/4 apart) and emit the wave's partial of
        // this item
        const int64_t pbase = (static_cast<int64_t>(it) * kDecodeWaves + wave) * RG;
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float tot = acc[c][i] + __shfl_down(acc[c][i], RP * 4, kWave);
                const int r = 4 * g4 + i;
                if (r < RG && ww.grp * RG + r < shp.rows_per_kv) part_acc[(pbase + r) * D + (c / (LANEB / 2)) * (8 * LANEB) + n16 * (LANEB / 2) + c % (LANEB / 2)] = tot;
            }
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const float l = wave_sum(l_lane[r]);
            if (lane == 0) {
                part_ml[(pbase + r) * 2] = m_run[r];
                part_ml[(pbase + r) * 2 + 1] = l;
            }
        }
    }
}

// ---- fp32 values: P.V on the vector ALUs --------------------------------------------------------
// The probabilities go through LDS to a mapping with 8 channels per lane; lanes with the same
// lane / (d / 8) walk the same keys.
template <class P, int RG>
struct DecodeSmemValu {
    DecodeTables<P> tb;
    float pbuf[kDecodeWaves][kWave][RG];
};

// VQ: the values are group-quantised rows (Sec. 4, "value-side group size"; the "value dequantization" of
// Alg. 2): per token [v_bits-bit codes, channel j at bit v_bits * j][per group of v_group channels: fp32
// scale, fp32 zero point], dequantised as zero + scale * code while they are accumulated.
template <class P, int RG, bool VQ = false>
__global__ __launch_bounds__(kDecodeWaves *kWave) void decode_kernel_valu(
    DeviceBooks books, DecodeShape shp, const float *__restrict__ q_rot, const uint4 *__restrict__ cache,
    const float4 *__restrict__ v, const int32_t *__restrict__ seq_lens, float *__restrict__ part_ml,
    float *__restrict__ part_acc, float *__restrict__ scores_out, int32_t *__restrict__ plan, int v_bits,
    int v_group) {
    constexpr int D = P::D;
    constexpr int LPR = D / 8;          // lanes per value row (8 channels per lane)
    constexpr int KPL = kWave / LPR;    // value rows per wave-wide load
    constexpr int TPS = decode_keys_per_lane<D>();  // tiles per step of the split sizing
    extern __shared__ __align__(16) unsigned char smem_raw[];
    DecodeSmemValu<P, RG> &sm = *reinterpret_cast<DecodeSmemValu<P, RG> *>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    build_tables<P>(sm.tb, books, tid, kDecodeWaves * kWave);
    __shared__ int item_slot;
    const int rl = lane % LPR, ko = lane / LPR;
    int it, taken = 0;
    while (next_item(plan, &item_slot, tid, &taken, &it)) {
    WaveWork ww;
    item_work(shp, plan, seq_lens, it, wave, TPS, &ww);
    const float *qg = q_rot + ww.group_id * (P::QS * RG);
    const uint4 *region = cache + ww.pair * (shp.t_capacity * P::GRANULES);
    const int64_t v_row0 = ww.pair * shp.t_capacity;

    float m_run[RG], l_lane[RG], acc[RG][8];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        m_run[r] = -INFINITY;
        l_lane[r] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[r][c] = 0.0f;
    }

    // the splits are sized in steps of TPS tiles (shared with the bf16-value kernel); here a step is
    // simply TPS tiles one after the other
    for (int step = ww.step_begin; step < ww.step_end; step += ww.step_stride)
    for (int tile = step * TPS; tile < min((step + 1) * TPS, ww.n_tiles); ++tile) {
        const int t0 = tile * kWave;
        const int n_valid = min(kWave, ww.len - t0);
        uint32_t w1[1][P::NWORDS];
        uint32_t (&w)[P::NWORDS] = w1[0];
        const uint4 *src = region + static_cast<int64_t>(tile) * (P::GRANULES * kWave) + lane;
#pragma unroll
        for (int g = 0; g < P::GRANULES; ++g) {
            typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
            const u32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + g * kWave));   // streamed
            w[4 * g] = x.x; w[4 * g + 1] = x.y; w[4 * g + 2] = x.z; w[4 * g + 3] = x.w;
        }
        // VQ: the tile's quantised value words are requested here, so that they arrive during the scores.
        // This lane's 8 channels of a row are 8 * v_bits bits at byte rl * v_bits, fetched as the two aligned
        // words around them (the second may reach into the row's own metadata); rows past the last token
        // are re-reads of the last one (their probabilities are zero).
        constexpr int NIT = VQ ? kWave / KPL : 1;   // key rows per lane and tile
        uint32_t q_lo[NIT], q_hi[NIT];
        float2 q_meta[NIT];
        if constexpr (VQ) {
            const int code_bytes = v_bits * (D / 8);
            const int row_bytes = code_bytes + (D / v_group) * 8;
            const int boff = rl * v_bits;
            const unsigned char *base = reinterpret_cast<const unsigned char *>(v) + (v_row0 + t0) * row_bytes;
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
                const unsigned char *row = base + static_cast<int64_t>(min(i * KPL + ko, n_valid - 1)) * row_bytes;
                const uint32_t *wp = reinterpret_cast<const uint32_t *>(row) + (boff >> 2);
                q_lo[i] = wp[0];
                q_hi[i] = wp[1];
                q_meta[i] = *reinterpret_cast<const float2 *>(row + code_bytes + ((rl * 8) / v_group) * 8);
            }
        }
        float s1[1][RG];
        float (&s)[RG] = s1[0];
        int q_off = 0;
        asm volatile("" : "+s"(q_off));
        tile_scores<P, RG, 1>(w1, qg + q_off, sm.tb, lane, s1);
        const float gamma = __uint_as_float(w[0]);
        const bool valid = lane < n_valid;
#pragma unroll
        for (int r = 0; r < RG; ++r) s[r] = valid ? s[r] * gamma : -INFINITY;
        if (scores_out != nullptr && valid) store_scores<RG>(shp, ww, scores_out, t0 + lane, s);
        float alpha[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const float m_new = fmaxf(m_run[r], wave_max(s[r]));
            alpha[r] = exp2_raw((m_run[r] - m_new) * kLog2e);
            m_run[r] = m_new;
            const float p = exp2_raw((s[r] - m_new) * kLog2e);
            l_lane[r] = fmaf(l_lane[r], alpha[r], p);
            sm.pbuf[wave][lane][r] = p;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] *= alpha[r];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if constexpr (VQ) {
            const uint32_t mask = (1u << v_bits) - 1u;
            const uint32_t sh = static_cast<uint32_t>((rl * v_bits) & 3);
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
                const int key = i * KPL + ko;           // probabilities of lanes past n_valid are zero
                float pv[RG];
#pragma unroll
                for (int r = 0; r < RG; ++r) pv[r] = sm.pbuf[wave][key][r];
                const uint32_t bits = __builtin_amdgcn_alignbyte(q_hi[i], q_lo[i], sh);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const float val = fmaf(q_meta[i].x, static_cast<float>((bits >> (c * v_bits)) & mask), q_meta[i].y);
#pragma unroll
                    for (int r = 0; r < RG; ++r) acc[r][c] = fmaf(pv[r], val, acc[r][c]);
                }
            }
        } else {
            for (int kb = 0; kb < n_valid; kb += KPL) {
                const int key = kb + ko;
                if (key < n_valid) {
                    float pv[RG];
#pragma unroll
                    for (int r = 0; r < RG; ++r) pv[r] = sm.pbuf[wave][key][r];
                    const int64_t vrow = v_row0 + t0 + key;
                    const float4 a = v[vrow * (D / 4) + 2 * rl];
                    const float4 b = v[vrow * (D / 4) + 2 * rl + 1];
                    const float vals[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int r = 0; r < RG; ++r)
#pragma unroll
                        for (int c = 0; c < 8; ++c) acc[r][c] = fmaf(pv[r], vals[c], acc[r][c]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // D7: fold the KPL lane groups and emit the wave's partial
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1)
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] += __shfl_xor(acc[r][c], o, kWave);
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const float l = wave_sum(l_lane[r]);
        const int64_t prow = (static_cast<int64_t>(it) * kDecodeWaves + wave) * RG + r;
        if (lane == 0) { part_ml[prow * 2] = m_run[r]; part_ml[prow * 2 + 1] = l; }
        if (ww.grp * RG + r >= shp.rows_per_kv) continue;
        if (ko == 0) {
#pragma unroll
            for (int c = 0; c < 8; ++c) part_acc[prow * D + rl * 8 + c] = acc[r][c];
        }
    }
    }   // items
}

// ---- D8: merge of the split partials, one wavefront per output row -----------------------------------
// out = sum_j w_j acc_j / sum_j w_j l_j with w_j = exp(m_j - max_j m_j) (the flash-decoding identity).
// A split without tokens has m = -inf, l = 0 and a zero accumulator, so it needs no special case.
template <int D>
__global__ __launch_bounds__(kWave) void merge_kernel(DecodeShape shp, const float *__restrict__ part_ml,
                                                      const float *__restrict__ part_acc,
                                                      const int32_t *__restrict__ plan, float *__restrict__ out,
                                                      const float *__restrict__ win_ml,
                                                      const float *__restrict__ win_acc) {
    // win_ml / win_acc (or NULL): one more partial per output row, that of a native-precision window
    constexpr int CPT = D / kWave;  // channels per lane
    constexpr int UN = 8;           // partial rows in flight per lane
    __shared__ float wgt[kWave];
    const int lane = threadIdx.x;
    const int64_t orow = blockIdx.x;  // (seq, qi, head)
    const int head = static_cast<int>(orow % shp.n_q_heads);
    const int qi = static_cast<int>((orow / shp.n_q_heads) % shp.n_q);
    const int seq = static_cast<int>(orow / (static_cast<int64_t>(shp.n_q_heads) * shp.n_q));
    const int kvh = head / shp.heads_per_kv;
    const int row = qi * shp.heads_per_kv + head % shp.heads_per_kv;
    const int grp = row / shp.rows_per_pass, r = row % shp.rows_per_pass;
    // Partial j of this row is at prow0 + j * pstride, j < n_part.  The many-row kernel (blocks of 128 or 256 rows):
    // one partial per split, adjacent.  Otherwise: the items of this row's (sequence, KV head, row group)
    // are consecutive, each with one partial per wavefront, RG rows apart.
    int64_t prow0;
    int n_part, pstride;
    if (plan == nullptr) {
        prow0 = (((static_cast<int64_t>(seq) * shp.n_kv_heads + kvh) * shp.n_row_groups + grp) * shp.rows_per_pass + r) *
                shp.n_splits;
        n_part = shp.n_splits;
        pstride = 1;
    } else {
        const int G = shp.n_kv_heads * shp.n_row_groups;
        const int before = plan[kPlanHeader + seq];
        const int c_s = (plan[kPlanHeader + seq + 1] - before) / G;
        const int64_t first = before + static_cast<int64_t>(kvh * shp.n_row_groups + grp) * c_s;
        prow0 = first * shp.item_waves * shp.rows_per_pass + r;
        n_part = c_s * shp.item_waves;
        pstride = shp.rows_per_pass;
    }
    // The first UN accumulator rows are requested before anything waits for the (m, l) pairs: their addresses do
    // not depend on them, and with the usual handful of partials per row this is all there is to read.
    float x_first[UN][CPT];
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
        for (int c = 0; c < CPT; ++c)
            x_first[u][c] = n_part > 0 ? part_acc[(prow0 + static_cast<int64_t>(min(u, n_part - 1)) * pstride) * D +
                                                  c * kWave + lane]
                                       : 0.0f;   // (an empty sequence has no partial)
    float m = -INFINITY;
    for (int j = lane; j < n_part; j += kWave) m = fmaxf(m, part_ml[(prow0 + static_cast<int64_t>(j) * pstride) * 2]);
    m = wave_max(m);
    if (win_ml != nullptr) m = fmaxf(m, win_ml[orow * 2]);
    float a[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) a[c] = 0.0f;
    float l = 0.0f;
    if (win_ml != nullptr) {
        const float mw = win_ml[orow * 2];
        const float f = (mw == -INFINITY) ? 0.0f : exp2_raw((mw - m) * kLog2e);
        if (lane == 0) l = f * win_ml[orow * 2 + 1];
#pragma unroll
        for (int c = 0; c < CPT; ++c) a[c] = f * win_acc[orow * D + c * kWave + lane];
    }
    for (int j0 = 0; j0 < n_part; j0 += kWave) {
        const int j = j0 + lane;
        float f = 0.0f;
        if (j < n_part) {
            const float2 ml = *reinterpret_cast<const float2 *>(part_ml + (prow0 + static_cast<int64_t>(j) * pstride) * 2);
            f = (ml.x == -INFINITY) ? 0.0f : exp2_raw((ml.x - m) * kLog2e);
            l += f * ml.y;
        }
        __syncthreads();
        wgt[lane] = f;
        __syncthreads();
        const int nj = min(kWave, n_part - j0);
        for (int jj = 0; jj < nj; jj += UN) {
            float x[UN][CPT];
            if (j0 == 0 && jj == 0) {
#pragma unroll
                for (int u = 0; u < UN; ++u)
#pragma unroll
                    for (int c = 0; c < CPT; ++c) x[u][c] = x_first[u][c];
            } else {
#pragma unroll
                for (int u = 0; u < UN; ++u)
#pragma unroll
                    for (int c = 0; c < CPT; ++c)
                        x[u][c] = part_acc[(prow0 + static_cast<int64_t>(j0 + min(jj + u, nj - 1)) * pstride) * D +
                                           c * kWave + lane];
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const float fj = (jj + u < nj) ? wgt[jj + u] : 0.0f;
#pragma unroll
                for (int c = 0; c < CPT; ++c) a[c] = fmaf(fj, x[u][c], a[c]);
            }
        }
    }
    l = wave_sum(l);
#pragma unroll
    for (int c = 0; c < CPT; ++c) out[orow * D + c * kWave + lane] = (l > 0.0f) ? a[c] / l : 0.0f;
}

// ---- launch helpers -----------------------------------------------------------------------------
template <class P>
int launch_decode_mq(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                     const void *v, const int32_t *seq_lens, float *part_ml, float *part_acc, hipStream_t stream,
                     PageTable pt = PageTable{nullptr, 0, 0});   // pt: cache and v are pools of pages

// bf16 values: the matrix-core kernels.  SCORES: the instantiation that also writes the scores (built in
// a translation unit of its own).
template <class P, int RG, bool SCORES>
int launch_decode_mfma_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                          const void *v, const int32_t *seq_lens, float *part_ml, float *part_acc, float *scores_out,
                          int32_t *plan, hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    // one workgroup per compute unit; they share the items of the plan
    hipLaunchKernelGGL((decode_kernel_mfma<P, RG, SCORES, false>), dim3(kDecodeWorkgroups), dim3(kDecodeWaves * kWave),
                       0, stream, books, s, q_rot, static_cast<const uint4 *>(cache), static_cast<const uint32_t *>(v),
                       seq_lens, part_ml, part_acc, scores_out, plan, nullptr, nullptr, nullptr, 0, 0);
    return static_cast<int>(hipGetLastError());
}

// Paged pools (bf16 values, row groups of at most 8 rows).
template <class P, int RG>
int launch_decode_paged_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *k_pool,
                           const void *v_pool, const PageTable &pt, const int32_t *seq_lens, float *part_ml,
                           float *part_acc, int32_t *plan, hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    hipLaunchKernelGGL((decode_kernel_mfma<P, RG, false, false, true>), dim3(kDecodeWorkgroups),
                       dim3(kDecodeWaves * kWave), 0, stream, books, s, q_rot, static_cast<const uint4 *>(k_pool),
                       static_cast<const uint32_t *>(v_pool), seq_lens, part_ml, part_acc, nullptr, plan, nullptr,
                       nullptr, pt.table, pt.stride, pt.n_pages);
    return static_cast<int>(hipGetLastError());
}

template <class P>
int launch_decode_paged_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                             const void *k_pool, const void *v_pool, const PageTable &pt, const int32_t *seq_lens,
                             float *part_ml, float *part_acc, int32_t *plan, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_paged_rg<P, 1>(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 2: return launch_decode_paged_rg<P, 2>(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 4: return launch_decode_paged_rg<P, 4>(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 8: return launch_decode_paged_rg<P, 8>(cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 128:
        case 256:   // the many-row kernel (d <= 128), which takes the page table as an argument
            if constexpr (P::D <= 128) return launch_decode_mq<P>(cb, s, q_rot, k_pool, v_pool, seq_lens, part_ml, part_acc, stream, pt);
            return static_cast<int>(hipErrorInvalidValue);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

// Paged pools with the QJL side-car in pages as well (a pool of [page][KV head] side-car tiles).
template <class P, int RG>
int launch_decode_paged_qjl_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                               const void *k_pool, const void *qjl_pool, const float *q2, const void *v_pool,
                               const PageTable &pt, const int32_t *seq_lens, float *part_ml, float *part_acc,
                               int32_t *plan, hipStream_t stream) {
    if constexpr (qjl_fits<P, RG>()) {
        const DeviceBooks books = device_books(cb);
        hipLaunchKernelGGL((decode_kernel_mfma<P, RG, true, true, true>), dim3(kDecodeWorkgroups),
                           dim3(kDecodeWaves * kWave), 0, stream, books, s, q_rot, static_cast<const uint4 *>(k_pool),
                           static_cast<const uint32_t *>(v_pool), seq_lens, part_ml, part_acc, nullptr, plan,
                           static_cast<const unsigned char *>(qjl_pool), q2, pt.table, pt.stride, pt.n_pages);
        return static_cast<int>(hipGetLastError());
    } else {
        return static_cast<int>(hipErrorInvalidValue);
    }
}

template <class P>
int launch_decode_paged_qjl_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                                 const void *k_pool, const void *qjl_pool, const float *q2, const void *v_pool,
                                 const PageTable &pt, const int32_t *seq_lens, float *part_ml, float *part_acc,
                                 int32_t *plan, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_paged_qjl_rg<P, 1>(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 2: return launch_decode_paged_qjl_rg<P, 2>(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 4: return launch_decode_paged_qjl_rg<P, 4>(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        case 8: return launch_decode_paged_qjl_rg<P, 8>(cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc, plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

template <class P, bool SCORES>
int launch_decode_mfma_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                            const void *cache, const void *v, const int32_t *seq_lens, float *part_ml,
                            float *part_acc, float *scores_out, int32_t *plan, hipStream_t stream) {
    if ((scores_out != nullptr) != SCORES) return static_cast<int>(hipErrorInvalidValue);
    switch (s.rows_per_pass) {
        case 1: return launch_decode_mfma_rg<P, 1, SCORES>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 2: return launch_decode_mfma_rg<P, 2, SCORES>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 4: return launch_decode_mfma_rg<P, 4, SCORES>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 8: return launch_decode_mfma_rg<P, 8, SCORES>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 128:
        case 256:   // the many-row kernel: 256 rows per workgroup at d = 64, 128 at d = 128
            if constexpr (P::D <= 128 && !SCORES)
                return launch_decode_mq<P>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, stream);
            return static_cast<int>(hipErrorInvalidValue);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

// fp32 values: P.V on the vector units
template <class P, int RG>
int launch_decode_valu_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                          const void *v, const int32_t *seq_lens, float *part_ml, float *part_acc, float *scores_out,
                          int32_t *plan, hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    const size_t smem = sizeof(DecodeSmemValu<P, RG>);
    const hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_kernel_valu<P, RG>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
    if (err != hipSuccess) return static_cast<int>(err);
    hipLaunchKernelGGL((decode_kernel_valu<P, RG>), dim3(kDecodeWorkgroups), dim3(kDecodeWaves * kWave), smem, stream,
                       books, s, q_rot, static_cast<const uint4 *>(cache), static_cast<const float4 *>(v), seq_lens,
                       part_ml, part_acc, scores_out, plan, 0, 0);
    return static_cast<int>(hipGetLastError());
}

template <class P>
int launch_decode_valu_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                            const void *cache, const void *v, const int32_t *seq_lens, float *part_ml,
                            float *part_acc, float *scores_out, int32_t *plan, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_valu_rg<P, 1>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 2: return launch_decode_valu_rg<P, 2>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 4: return launch_decode_valu_rg<P, 4>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 8: return launch_decode_valu_rg<P, 8>(cb, s, q_rot, cache, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

// Decode attention over group-quantised values.
template <class P, int RG>
int launch_decode_vq_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                        const void *vq, int v_bits, int v_group, const int32_t *seq_lens, float *part_ml,
                        float *part_acc, float *scores_out, int32_t *plan, hipStream_t stream) {
    const DeviceBooks books = device_books(cb);
    const size_t smem = sizeof(DecodeSmemValu<P, RG>);
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_kernel_valu<P, RG, true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
    if (err != hipSuccess) return static_cast<int>(err);
    hipLaunchKernelGGL((decode_kernel_valu<P, RG, true>), dim3(kDecodeWorkgroups), dim3(kDecodeWaves * kWave), smem,
                       stream, books, s, q_rot, static_cast<const uint4 *>(cache), static_cast<const float4 *>(vq),
                       seq_lens, part_ml, part_acc, scores_out, plan, v_bits, v_group);
    return static_cast<int>(hipGetLastError());
}

template <class P>
int launch_decode_vq_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                          const void *vq, int v_bits, int v_group, const int32_t *seq_lens, float *part_ml,
                          float *part_acc, float *scores_out, int32_t *plan, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_vq_rg<P, 1>(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 2: return launch_decode_vq_rg<P, 2>(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 4: return launch_decode_vq_rg<P, 4>(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 8: return launch_decode_vq_rg<P, 8>(cb, s, q_rot, cache, vq, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

// Largest row group whose sign-byte table fits LDS beside the codebook tables (8 at d = 64, 4 at
// d = 128, 2 at d = 256).
template <class P, int RG>
int launch_decode_qjl_rg(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot, const void *cache,
                         const void *qjl, const float *q2, const void *v, const int32_t *seq_lens, float *part_ml,
                         float *part_acc, float *scores_out, int32_t *plan, hipStream_t stream) {
    if constexpr (qjl_fits<P, RG>()) {
        const DeviceBooks books = device_books(cb);
        hipLaunchKernelGGL((decode_kernel_mfma<P, RG, true, true>), dim3(kDecodeWorkgroups),
                           dim3(kDecodeWaves * kWave), 0, stream, books, s, q_rot, static_cast<const uint4 *>(cache),
                           static_cast<const uint32_t *>(v), seq_lens, part_ml, part_acc, scores_out, plan,
                           static_cast<const unsigned char *>(qjl), q2, nullptr, 0, 0);
        return static_cast<int>(hipGetLastError());
    } else {
        return static_cast<int>(hipErrorInvalidValue);
    }
}

template <class P>
int launch_decode_qjl_plan(const octopus_codebooks_t &cb, const DecodeShape &s, const float *q_rot,
                           const void *cache, const void *qjl, const float *q2, const void *v,
                           const int32_t *seq_lens, float *part_ml, float *part_acc, float *scores_out,
                           int32_t *plan, hipStream_t stream) {
    switch (s.rows_per_pass) {
        case 1: return launch_decode_qjl_rg<P, 1>(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 2: return launch_decode_qjl_rg<P, 2>(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 4: return launch_decode_qjl_rg<P, 4>(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        case 8: return launch_decode_qjl_rg<P, 8>(cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, plan, stream);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace octopus

#endif
