// Host side of the OCTOPUS library: plan (Sec. 3.2-3.3), Lloyd-Max codebooks
// (Sec. 3.4), argument validation and launch dispatch for the C ABI.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include <hip/hip_runtime.h>

#include "octopus_internal.h"

namespace octopus {
namespace {

// ---- numerical integration ------------------------------------------------------------------
// Composite 16-point Gauss-Legendre; nodes from Newton's iteration on the Legendre polynomial.
struct GaussLegendre16 {
    static constexpr int N = 16;
    double x[N], w[N];
    GaussLegendre16() {
        const double pi = std::acos(-1.0);
        for (int i = 0; i < N; ++i) {
            double z = std::cos(pi * (i + 0.75) / (N + 0.5));
            double dp = 0.0;
            for (int it = 0; it < 100; ++it) {
                double p0 = 1.0, p1 = z;
                for (int k = 2; k <= N; ++k) {
                    double p2 = ((2.0 * k - 1.0) * z * p1 - (k - 1.0) * p0) / k;
                    p0 = p1;
                    p1 = p2;
                }
                dp = N * (z * p1 - p0) / (z * z - 1.0);
                double dz = p1 / dp;
                z -= dz;
                if (std::fabs(dz) < 1e-16) break;
            }
            x[i] = z;
            w[i] = 2.0 / ((1.0 - z * z) * dp * dp);
        }
    }
};

const GaussLegendre16 &gl() {
    static const GaussLegendre16 g;
    return g;
}

// integral over [a, b] of f(t) and of t * f(t)
template <class F>
void mass_and_moment(const F &f, double a, double b, int panels, double *mass, double *moment) {
    const GaussLegendre16 &g = gl();
    double m = 0.0, mx = 0.0;
    const double h = (b - a) / panels;
    for (int p = 0; p < panels; ++p) {
        const double mid = a + (p + 0.5) * h, half = 0.5 * h;
        for (int i = 0; i < GaussLegendre16::N; ++i) {
            const double t = mid + half * g.x[i];
            const double ft = f(t) * g.w[i] * half;
            m += ft;
            mx += ft * t;
        }
    }
    *mass = m;
    *moment = mx;
}

// Lloyd-Max quantiser of density f on [lo, hi]: alternate "boundaries = midpoints of adjacent
// centroids" and "centroids = conditional means" to the fixed point, from the equal-probability
// quantiles F^-1((k + 1/2) / levels).
template <class F>
std::vector<double> lloyd_max(const F &f, int levels, double lo, double hi) {
    double total, unused;
    mass_and_moment(f, lo, hi, 256, &total, &unused);
    std::vector<double> c(levels);
    for (int k = 0; k < levels; ++k) {
        const double target = total * (k + 0.5) / levels;
        double a = lo, b = hi;
        for (int it = 0; it < 200; ++it) {
            const double mid = 0.5 * (a + b);
            double m;
            mass_and_moment(f, lo, mid, 64, &m, &unused);
            if (m < target) a = mid; else b = mid;
        }
        c[k] = 0.5 * (a + b);
    }
    std::vector<double> edge(levels + 1);
    for (int it = 0; it < 400000; ++it) {
        edge[0] = lo;
        edge[levels] = hi;
        for (int k = 1; k < levels; ++k) edge[k] = 0.5 * (c[k - 1] + c[k]);
        double move = 0.0;
        for (int k = 0; k < levels; ++k) {
            double m, mx;
            mass_and_moment(f, edge[k], edge[k + 1], 8, &m, &mx);
            const double cn = mx / m;
            move = std::max(move, std::fabs(cn - c[k]));
            c[k] = cn;
        }
        if (move < 1e-13) break;
    }
    return c;
}

// Eq. (rho-pdf)
struct RhoDensity {
    double expo, norm;
    explicit RhoDensity(int d) : expo(0.5 * (d - 5)) {
        const double a = 1.5, b = 0.5 * (d - 3);
        norm = 2.0 / std::exp(std::lgamma(a) + std::lgamma(b) - std::lgamma(a + b));
    }
    double operator()(double r) const {
        const double one_minus = 1.0 - r * r;
        return one_minus <= 0.0 ? 0.0 : norm * r * r * std::pow(one_minus, expo);
    }
};

// Eq. (oct-marginal), folded onto a = |xi| in [0, 1] (density doubled)
struct XiHalfDensity {
    double operator()(double a) const {
        const double pi = std::acos(-1.0);
        const double lead = 1.0 / (pi * std::sqrt(a * a + (1.0 - a) * (1.0 - a)));
        return 2.0 * lead * ((1.0 - a) / (1.0 - 2.0 * a + 3.0 * a * a) + a / (2.0 - 4.0 * a + 3.0 * a * a));
    }
};

std::mutex g_book_mutex;
std::map<int, std::vector<float>> g_xi_books;                  // key: b_dir
std::map<std::pair<int, int>, std::vector<float>> g_rho_books; // key: (d, b_nrm)

std::vector<float> xi_centroids(int b_dir) {
    std::lock_guard<std::mutex> lock(g_book_mutex);
    auto it = g_xi_books.find(b_dir);
    if (it != g_xi_books.end()) return it->second;
    const int levels = 1 << b_dir, half = levels / 2;
    std::vector<double> pos = lloyd_max(XiHalfDensity(), half, 0.0, 1.0);
    std::vector<float> c(levels);
    for (int k = 0; k < half; ++k) {
        c[half + k] = static_cast<float>(pos[k]);
        c[half - 1 - k] = -static_cast<float>(pos[k]);
    }
    g_xi_books[b_dir] = c;
    return c;
}

std::vector<float> rho_centroids(int d, int b_nrm) {
    std::lock_guard<std::mutex> lock(g_book_mutex);
    auto key = std::make_pair(d, b_nrm);
    auto it = g_rho_books.find(key);
    if (it != g_rho_books.end()) return it->second;
    std::vector<double> c64 = lloyd_max(RhoDensity(d), 1 << b_nrm, 0.0, 1.0);
    std::vector<float> c(c64.begin(), c64.end());
    g_rho_books[key] = c;
    return c;
}

void midpoints(const float *c, int levels, float *b) {
    for (int k = 0; k + 1 < levels; ++k)
        b[k] = static_cast<float>(0.5 * (static_cast<double>(c[k]) + static_cast<double>(c[k + 1])));
}

int gcd_int(int a, int b) { return b == 0 ? a : gcd_int(b, a % b); }

// Stream of n indices of b bits; the count is padded to whole byte groups (the sizes the KV
// ratios of the paper's kernel-speed table imply).
int stream_bytes(int n, int b) {
    const int g = 8 / gcd_int(b, 8);
    return ((n + g - 1) / g) * (g * b / 8);
}

bool head_dim_ok(int d) { return d == 64 || d == 128 || d == 256; }

// Sec. 3.3: implemented split around nominal b; b = 1 -> (1, 1).
bool split_of(int b, int *b_dir, int *b_nrm) {
    if (b == 1) { *b_dir = 1; *b_nrm = 1; return true; }
    if (b >= 2 && b <= 4) { *b_dir = b + 1; *b_nrm = b - 1; return true; }
    return false;
}

void finish_plan(octopus_plan_t *p) {
    p->dir_bytes = 0;
    p->nrm_bytes = 0;
    for (int c = 0; c < p->n_class; ++c) {
        p->dir_bytes += stream_bytes(2 * p->class_ntri[c], p->b_dir[c]);
        p->nrm_bytes += stream_bytes(p->class_ntri[c], p->b_nrm[c]);
    }
    p->record_bytes = 4 + p->dir_bytes + p->nrm_bytes;
    p->granules = (p->record_bytes + 15) / 16;
}

void fill_books(octopus_codebooks_t *out) {
    const octopus_plan_t &p = out->plan;
    for (int c = 0; c < p.n_class; ++c) {
        std::vector<float> cx = xi_centroids(p.b_dir[c]);
        std::vector<float> cr = rho_centroids(p.head_dim, p.b_nrm[c]);
        std::copy(cx.begin(), cx.end(), out->c_xi[c]);
        std::copy(cr.begin(), cr.end(), out->c_rho[c]);
        midpoints(out->c_xi[c], 1 << p.b_dir[c], out->b_xi[c]);
        midpoints(out->c_rho[c], 1 << p.b_nrm[c], out->b_rho[c]);
    }
}

bool plan_consistent(const octopus_plan_t &p) {
    if (!head_dim_ok(p.head_dim) || p.n_tri != (p.head_dim + 2) / 3) return false;
    if (p.n_class < 1 || p.n_class > 2) return false;
    int total = 0;
    for (int c = 0; c < p.n_class; ++c) {
        if (p.class_ntri[c] < 1 || p.b_dir[c] < 1 || p.b_dir[c] > 6 || p.b_nrm[c] < 1 || p.b_nrm[c] > 6) return false;
        total += p.class_ntri[c];
    }
    if (total != p.n_tri) return false;
    octopus_plan_t q = p;
    finish_plan(&q);
    return q.dir_bytes == p.dir_bytes && q.nrm_bytes == p.nrm_bytes && q.record_bytes == p.record_bytes &&
           q.granules == p.granules;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

DecodeShape make_decode_shape(const octopus_plan_t &plan, int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t n_q, int64_t max_len, int64_t t_capacity, bool many_rows, int32_t rows_cap,
                              int32_t vq_mfma_waves) {
    DecodeShape s{};
    s.n_seq = n_seq;
    s.n_q_heads = n_q_heads;
    s.n_kv_heads = n_kv_heads;
    s.n_q = n_q;
    s.heads_per_kv = n_q_heads / n_kv_heads;
    s.rows_per_kv = n_q * s.heads_per_kv;
    s.t_capacity = t_capacity;
    s.max_len = static_cast<int32_t>(max_len);
    s.item_waves = 4;
    s.tiles_per_step = plan.head_dim <= 128 ? 2 : 1;
    const int64_t len = std::max<int64_t>(max_len, 1);
    if (many_rows) {
        // Matrix-core kernel for many query rows: blocks of 128 rows (4 wavefronts), or of 256 rows (8
        // wavefronts) at d = 64 when there are rows enough; one workgroup per (block, split).  A compute unit
        // runs 8 of these wavefronts at d = 64 and 4 at d = 128.
        s.rows_per_pass = (plan.head_dim <= 64 && s.rows_per_kv >= 192) ? 256 : 128;
        s.n_row_groups = (s.rows_per_kv + s.rows_per_pass - 1) / s.rows_per_pass;
        const int64_t groups = static_cast<int64_t>(n_seq) * n_kv_heads * s.n_row_groups;
        const int64_t max_tiles = (len + OCTOPUS_TILE - 1) / OCTOPUS_TILE;
        const int64_t slots = (plan.head_dim <= 64 && s.rows_per_pass == 128) ? 512 : 256;
        // The workgroups run in rounds of `slots`.  Among the split counts (each split keeping at least 16 tiles)
        // the fullest last round wins, but every split writes a partial result per query row that the merge reads
        // again: the smallest count within 3 % of the best fill is taken (the Lumiere-shaped batch: 7 splits
        // at 98.4 % instead of 32 at 100 %, a fifth of the partial traffic).
        auto fill = [&](int64_t n) {
            const int64_t wgs = groups * n, rounds = (wgs + slots - 1) / slots;
            return static_cast<double>(wgs) / static_cast<double>(rounds * slots);
        };
        double best_eff = 0.0;
        for (int64_t n = 1; n <= 32 && (n == 1 || max_tiles / n >= 16); ++n) best_eff = std::max(best_eff, fill(n));
        int64_t best = 1;
        for (int64_t n = 1; n <= 32 && (n == 1 || max_tiles / n >= 16); ++n)
            if (fill(n) >= best_eff - 0.03) { best = n; break; }
        s.n_splits = static_cast<int32_t>(best);
        return s;
    }
    // Query rows scored per key by one workgroup: the power of two covering rows_per_kv, at most 8
    // (fewer with the QJL residual).  Rows beyond rows_per_kv in the last group are zero queries whose
    // results are not stored.
    s.rows_per_pass = 1;
    while (s.rows_per_pass < s.rows_per_kv && s.rows_per_pass < rows_cap) s.rows_per_pass *= 2;
    if (vq_mfma_waves > 0) {
        // The matrix-core kernel over quantised values: row groups of 4 or 8; up to d = 128 two wavefronts per
        // SIMD (8 per workgroup) where their LDS fits, each taking one tile per step.
        s.rows_per_pass = vq_mfma_rows(s.rows_per_kv);
        s.tiles_per_step = 1;
        s.item_waves = vq_mfma_waves;
    }
    s.n_row_groups = (s.rows_per_kv + s.rows_per_pass - 1) / s.rows_per_pass;
    // Split-K sizing: one wavefront per split.  The decode kernel runs one wavefront per SIMD, 256
    // compute units x 4 at once; the steps (128 keys up to d = 128, 64 keys at d = 256) of each
    // (sequence, KV head, row group) are divided over as many splits as fill those slots once, so that
    // all wavefronts start together and end together.
    const int64_t groups = static_cast<int64_t>(n_seq) * n_kv_heads * s.n_row_groups;
    const int64_t step_keys = OCTOPUS_TILE * s.tiles_per_step;
    const int64_t max_steps = (len + step_keys - 1) / step_keys;
    const int64_t slots = 256 * 4;
    // workgroups of 4 wavefronts: splits come in fours
    int64_t want = (slots / 4 + groups / 2) / groups;
    want = std::max<int64_t>(1, std::min<int64_t>(want, (max_steps + 3) / 4));
    s.n_splits = static_cast<int32_t>(4 * want);   // kept for reference; the device cuts the items itself
    // The device cuts the work into at most 256 * 8 items plus one more per (sequence, KV head, row group)
    // (the rounding of each one's share), see the plan in the kernels.
    s.max_items = static_cast<int32_t>(std::min<int64_t>(256 * 8 + groups, groups * std::max<int64_t>(max_steps, 1)));
    return s;
}

// The matrix-core kernel for many query rows serves bf16 values without score output at d <= 128.
bool many_rows_shape(const octopus_plan_t &plan, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q) {
    return plan.head_dim <= 128 && static_cast<int64_t>(n_q) * (n_q_heads / n_kv_heads) >= 32;
}

Workspace make_workspace(const octopus_plan_t &plan, const DecodeShape &s) {
    auto up = [](size_t x) { return (x + 255) & ~static_cast<size_t>(255); };
    Workspace w{};
    const size_t rows = static_cast<size_t>(s.n_seq) * s.n_kv_heads * s.n_row_groups * s.rows_per_pass;
    // partial results: one per (row, split) with blocks of 128 or 256 rows, else one per (item, wavefront, row of
    // the group)
    const size_t partials = s.rows_per_pass >= 128 ? rows * s.n_splits
                                                   : static_cast<size_t>(s.max_items) * s.item_waves * s.rows_per_pass;
    w.q_rot_off = 0;
    const size_t q_bytes = up(rows * q_row_stride(plan.n_tri) * sizeof(float));
    w.part_ml_off = q_bytes;
    const size_t ml_bytes = up(partials * 2 * sizeof(float));
    w.part_acc_off = w.part_ml_off + ml_bytes;
    const size_t acc_bytes = up(partials * static_cast<size_t>(plan.head_dim) * sizeof(float));
    w.plan_off = w.part_acc_off + acc_bytes;
    const size_t plan_bytes = up((static_cast<size_t>(s.n_seq) + 5) * sizeof(int32_t));
    w.q2_off = w.plan_off + plan_bytes;   // second rotation of the queries (QJL residual only)
    w.win_ml_off = w.q2_off + up(rows * static_cast<size_t>(plan.head_dim) * sizeof(float));
    // partial of a native-precision window, one per output row (hybrid cache only)
    const size_t out_rows = static_cast<size_t>(s.n_seq) * s.n_q * s.n_q_heads;
    w.win_acc_off = w.win_ml_off + up(out_rows * 2 * sizeof(float));
    w.total = w.win_acc_off + up(out_rows * static_cast<size_t>(plan.head_dim) * sizeof(float));
    return w;
}

}  // namespace octopus

using namespace octopus;

namespace {
thread_local void *g_event_before = nullptr;
thread_local void *g_event_after = nullptr;
}  // namespace

extern "C" {

int octopus_profile_events(void *before, void *after) {
    if ((before == nullptr) != (after == nullptr)) return OCTOPUS_EINVAL;
    g_event_before = before;
    g_event_after = after;
    return OCTOPUS_OK;
}

int octopus_probe_read(const void *data, size_t bytes, int32_t nontemporal, int32_t n_workgroups, void *sink,
                       void *stream) {
    if (data == nullptr || sink == nullptr || !aligned(data, 16) || !aligned(sink, 4)) return OCTOPUS_EINVAL;
    if (n_workgroups < 1 || n_workgroups > (1 << 20) || bytes / 16 / static_cast<size_t>(n_workgroups) < 1)
        return OCTOPUS_EINVAL;
    const int err = launch_probe_read(data, static_cast<int64_t>(bytes), nontemporal != 0, n_workgroups, sink, stream);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_build_codebooks(int32_t head_dim, float bits, octopus_codebooks_t *out) {
    if (out == nullptr) return OCTOPUS_EINVAL;
    if (!head_dim_ok(head_dim)) return OCTOPUS_EUNSUPPORTED;
    const float twice_f = 2.0f * bits;
    const int twice = static_cast<int>(std::lround(twice_f));
    if (!(std::fabs(twice_f - twice) < 1e-6f) || twice < 2 || twice > 8) return OCTOPUS_EUNSUPPORTED;
    if (twice == 7) return OCTOPUS_EUNSUPPORTED;  // 3.5 is not one of the built widths
    std::memset(out, 0, sizeof(*out));
    octopus_plan_t &p = out->plan;
    p.head_dim = head_dim;
    p.n_tri = (head_dim + 2) / 3;
    if (twice % 2 == 0) {
        p.n_class = 1;
        p.class_ntri[0] = p.n_tri;
        if (!split_of(twice / 2, &p.b_dir[0], &p.b_nrm[0])) return OCTOPUS_EUNSUPPORTED;
    } else {
        p.n_class = 2;
        p.class_ntri[0] = (p.n_tri + 1) / 2;
        p.class_ntri[1] = p.n_tri - p.class_ntri[0];
        if (!split_of((twice + 1) / 2, &p.b_dir[0], &p.b_nrm[0])) return OCTOPUS_EUNSUPPORTED;
        if (!split_of((twice - 1) / 2, &p.b_dir[1], &p.b_nrm[1])) return OCTOPUS_EUNSUPPORTED;
    }
    finish_plan(&p);
    fill_books(out);
    return OCTOPUS_OK;
}

int octopus_build_codebooks_pair(int32_t head_dim, int32_t b_dir, int32_t b_nrm, octopus_codebooks_t *out) {
    if (out == nullptr) return OCTOPUS_EINVAL;
    if (!head_dim_ok(head_dim) || b_dir < 1 || b_dir > 6 || b_nrm < 1 || b_nrm > 6) return OCTOPUS_EUNSUPPORTED;
    std::memset(out, 0, sizeof(*out));
    octopus_plan_t &p = out->plan;
    p.head_dim = head_dim;
    p.n_tri = (head_dim + 2) / 3;
    p.n_class = 1;
    p.class_ntri[0] = p.n_tri;
    p.b_dir[0] = b_dir;
    p.b_nrm[0] = b_nrm;
    finish_plan(&p);
    fill_books(out);
    return OCTOPUS_OK;
}

size_t octopus_cache_bytes(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_kv_heads, int64_t t_capacity) {
    if (cb == nullptr || n_seq < 1 || n_kv_heads < 1 || t_capacity < OCTOPUS_TILE || t_capacity % OCTOPUS_TILE != 0)
        return 0;
    if (!plan_consistent(cb->plan)) return 0;
    return static_cast<size_t>(n_seq) * n_kv_heads * static_cast<size_t>(t_capacity) * cb->plan.granules * 16;
}

// The encoder finds the scalar seed through a grid of 8 * 2^b_dir cells over [-1, 1] and one compare; that
// is exact when no cell holds two boundaries of C_xi (true of every Lloyd-Max codebook this library builds;
// a caller-edited codebook may violate it).  Same fp32 arithmetic as the kernel.
// The encoder's direction table covers one quadrant of the code grid and relies on C_xi being antisymmetric,
// C_xi[K - 1 - k] == -C_xi[k] bit for bit, as the Lloyd-Max codebook of a symmetric marginal is (and every
// codebook this library builds).
static bool seed_grid_ok(const octopus_codebooks_t &cb) {
    for (int c = 0; c < cb.plan.n_class; ++c) {
        const int K = 1 << cb.plan.b_dir[c];
        for (int k = 0; k < K; ++k)
            if (!(cb.c_xi[c][K - 1 - k] == -cb.c_xi[c][k])) return false;
        const int ncell = 8 * K;
        int last = -1;
        for (int k = 0; k + 1 < K; ++k) {
            if (!(cb.c_xi[c][k] < cb.c_xi[c][k + 1])) return false;
            const float b = 0.5f * (cb.c_xi[c][k] + cb.c_xi[c][k + 1]);
            int cell = static_cast<int>(std::floor((b + 1.0f) * (0.5f * static_cast<float>(ncell))));
            cell = std::min(std::max(cell, 0), ncell - 1);
            if (cell <= last) return false;
            last = cell;
        }
    }
    return true;
}

static int encode_checked(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                          int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                          const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                          const uint8_t *signs2, void *qjl, void *stream, int32_t rounding = OCTOPUS_ROUND_LOCAL_3X3) {
    if (cb == nullptr || keys == nullptr || signs == nullptr || cache == nullptr) return OCTOPUS_EINVAL;
    if (rounding < OCTOPUS_ROUND_SEED || rounding > OCTOPUS_ROUND_LOCAL_2X2) return OCTOPUS_EINVAL;
    if (n_seq < 1 || n_kv_heads < 1 || n_new < 0) return OCTOPUS_EINVAL;
    if (n_seq > 65535 || n_kv_heads > 65535) return OCTOPUS_EINVAL;   // they are grid dimensions of the launch
    if (t_capacity < OCTOPUS_TILE || t_capacity % OCTOPUS_TILE != 0) return OCTOPUS_EINVAL;
    if (!plan_consistent(cb->plan)) return OCTOPUS_EINVAL;
    if (key_dtype != OCTOPUS_DTYPE_F32 && key_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
    // a pair of the App. D sweep has the plain encoder only (local 3x3, no side-car)
    const bool sweep = !plan_supported(cb->plan) && plan_sweep_only(cb->plan);
    if (sweep && (rounding != OCTOPUS_ROUND_LOCAL_3X3 || qjl != nullptr)) return OCTOPUS_EUNSUPPORTED;
    if ((!plan_supported(cb->plan) && !sweep) || !seed_grid_ok(*cb)) return OCTOPUS_EUNSUPPORTED;
    if (stride_seq < 0 || stride_tok < 0 || stride_head < 0) return OCTOPUS_EINVAL;
    if (stride_seq % 8 != 0 || stride_tok % 8 != 0 || stride_head % 8 != 0) return OCTOPUS_EINVAL;
    if (!aligned(keys, 16) || !aligned(cache, 16)) return OCTOPUS_EINVAL;
    if (qjl != nullptr && !aligned(qjl, 4)) return OCTOPUS_EINVAL;
    if (start_pos == nullptr && n_new > t_capacity) return OCTOPUS_EINVAL;
    if (n_new == 0) return OCTOPUS_OK;
    const int err = rounding == OCTOPUS_ROUND_LOCAL_3X3
                        ? launch_encode(*cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads,
                                        n_new, signs, cache, t_capacity, start_pos, signs2, qjl, stream)
                        : launch_encode_rounding(*cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq,
                                                 n_kv_heads, n_new, signs, cache, t_capacity, start_pos, rounding,
                                                 stream);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_encode(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                   int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                   const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos, void *stream) {
    return encode_checked(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs,
                          cache, t_capacity, start_pos, nullptr, nullptr, stream);
}

int octopus_encode_rounding(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                            int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                            const uint8_t *signs, void *cache, int64_t t_capacity, const int32_t *start_pos,
                            int32_t rounding, void *stream) {
    return encode_checked(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs,
                          cache, t_capacity, start_pos, nullptr, nullptr, stream, rounding);
}

size_t octopus_qjl_bytes(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_kv_heads, int64_t t_capacity) {
    if (cb == nullptr || n_seq < 1 || n_kv_heads < 1 || t_capacity < OCTOPUS_TILE || t_capacity % OCTOPUS_TILE != 0)
        return 0;
    if (!plan_consistent(cb->plan)) return 0;
    return static_cast<size_t>(n_seq) * n_kv_heads * static_cast<size_t>(t_capacity) * (cb->plan.head_dim / 8 + 2);
}

int octopus_encode_qjl(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                       int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                       const uint8_t *signs, const uint8_t *signs2, void *cache, void *qjl, int64_t t_capacity,
                       const int32_t *start_pos, void *stream) {
    if (signs2 == nullptr || qjl == nullptr) return OCTOPUS_EINVAL;
    return encode_checked(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs,
                          cache, t_capacity, start_pos, signs2, qjl, stream);
}

static int decode_args_ok(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t n_q, int64_t max_len) {
    if (cb == nullptr) return OCTOPUS_EINVAL;
    if (n_seq < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q < 1 || max_len < 0 || max_len > INT32_MAX)
        return OCTOPUS_EINVAL;
    if (n_q_heads % n_kv_heads != 0) return OCTOPUS_EINVAL;
    if (!plan_consistent(cb->plan)) return OCTOPUS_EINVAL;
    if (!plan_supported(cb->plan) && !plan_sweep_only(cb->plan)) return OCTOPUS_EUNSUPPORTED;
    return OCTOPUS_OK;
}

int octopus_vq_on_matrix_cores(const octopus_codebooks_t *cb, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q,
                               int32_t v_bits, int32_t v_group) {
    if (decode_args_ok(cb, 1, n_q_heads, n_kv_heads, n_q, 1) != OCTOPUS_OK) return 0;
    if (v_bits < 2 || v_bits > 4 || (v_group != 16 && v_group != 32)) return 0;
    return vq_mfma_available(cb->plan, vq_mfma_rows(n_q * (n_q_heads / n_kv_heads)), v_bits, v_group) > 0 ? 1 : 0;
}

// Workspace of a decode call without quantised values (what octopus_attn_decode_static has to fit).
static size_t plain_decode_workspace(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_q_heads,
                                     int32_t n_kv_heads, int32_t n_q, int64_t max_len) {
    const DecodeShape s = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, 0, false);
    size_t total = make_workspace(cb->plan, s).total;
    if (many_rows_shape(cb->plan, n_q_heads, n_kv_heads, n_q)) {   // the larger of the two kernels' needs
        const DecodeShape m = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, 0, true);
        total = std::max(total, make_workspace(cb->plan, m).total);
    }
    // ... and of the kernel with the QJL residual, which serves smaller row groups
    const int cap = qjl_rows_cap(cb->plan);
    if (cap > 0) {
        const DecodeShape j = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, 0, false, cap);
        total = std::max(total, make_workspace(cb->plan, j).total);
    }
    return total;
}

size_t octopus_attn_decode_workspace(const octopus_codebooks_t *cb, int32_t n_seq, int32_t n_q_heads,
                                     int32_t n_kv_heads, int32_t n_q, int64_t max_len) {
    if (decode_args_ok(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len) != OCTOPUS_OK) return 0;
    size_t total = plain_decode_workspace(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len);
    // ... and of the matrix-core kernel over quantised values (row groups of 4 or 8, up to 8 wavefronts an item)
    const DecodeShape vqs = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, 0, false, 8,
                                              cb->plan.head_dim <= 128 ? 8 : 4);
    total = std::max(total, make_workspace(cb->plan, vqs).total);
    return total;
}

namespace {
// Native-precision window of a hybrid cache (all NULL / 0: none).
struct WindowArgs {
    const void *k_window = nullptr;
    int32_t k_dtype = 0;
    int64_t w_capacity = 0;
    const int32_t *win_lens = nullptr;
};
}  // namespace

static int attn_decode(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                       int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs, const void *cache,
                       int64_t t_capacity, const void *v, int32_t v_dtype, const int32_t *seq_lens, int64_t max_len,
                       float scale, float *out, float *scores_out, void *workspace, size_t workspace_bytes,
                       void *stream, bool with_qjl, const uint8_t *signs2, const void *qjl, int v_bits = 0,
                       int v_group = 0, const WindowArgs *win = nullptr, bool static_scratch_call = false) {
    const bool with_vq = v_bits != 0;    // v: group-quantised rows (v_dtype is not looked at)
    // the measurement events belong to THIS call whatever becomes of it: a call that fails leaves none armed
    void *ev_before = g_event_before, *ev_after = g_event_after;
    g_event_before = g_event_after = nullptr;
    const int ok = decode_args_ok(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len);
    if (ok != OCTOPUS_OK) return ok;
    if (with_vq) {
        if (v_bits < 2 || v_bits > 4 || (v_group != 16 && v_group != 32)) return OCTOPUS_EUNSUPPORTED;
        v_dtype = OCTOPUS_DTYPE_F32;     // served by the kernel that accumulates on the vector units
    }
    if (q == nullptr || signs == nullptr || cache == nullptr || v == nullptr || seq_lens == nullptr || out == nullptr)
        return OCTOPUS_EINVAL;
    if (with_qjl && (signs2 == nullptr || qjl == nullptr)) return OCTOPUS_EINVAL;
    // a pair of the App. D sweep has the split-K kernel over bf16 values only
    const bool sweep = !plan_supported(cb->plan);
    if (sweep && (with_qjl || with_vq || v_dtype != OCTOPUS_DTYPE_BF16 || scores_out != nullptr ||
                  many_rows_shape(cb->plan, n_q_heads, n_kv_heads, n_q)))
        return OCTOPUS_EUNSUPPORTED;
    if (t_capacity < OCTOPUS_TILE || t_capacity % OCTOPUS_TILE != 0 || max_len > t_capacity) return OCTOPUS_EINVAL;
    if ((q_dtype != OCTOPUS_DTYPE_F32 && q_dtype != OCTOPUS_DTYPE_BF16) ||
        (v_dtype != OCTOPUS_DTYPE_F32 && v_dtype != OCTOPUS_DTYPE_BF16))
        return OCTOPUS_EUNSUPPORTED;
    if (with_qjl && v_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
    if (!aligned(cache, 16) || !aligned(v, 16) || !aligned(q, 4) || !aligned(out, 4)) return OCTOPUS_EINVAL;
    if (with_qjl && !aligned(qjl, 4)) return OCTOPUS_EINVAL;
    if (!std::isfinite(scale)) return OCTOPUS_EINVAL;
    if (win != nullptr) {
        if (win->k_window == nullptr || win->win_lens == nullptr || win->w_capacity < 1) return OCTOPUS_EINVAL;
        if (win->k_dtype != OCTOPUS_DTYPE_F32 && win->k_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
        if (!aligned(win->k_window, 16)) return OCTOPUS_EINVAL;
    }
    const bool many_rows = !with_qjl && !with_vq && many_rows_shape(cb->plan, n_q_heads, n_kv_heads, n_q) &&
                           v_dtype == OCTOPUS_DTYPE_BF16 && scores_out == nullptr;
    const int rows_cap = with_qjl ? qjl_rows_cap(cb->plan) : 8;
    if (rows_cap <= 0) return OCTOPUS_EUNSUPPORTED;
    // quantised values without score output: the matrix-core kernel where one is built for the shape
    const int32_t vq_mfma = with_vq && scores_out == nullptr
                                ? vq_mfma_available(cb->plan, vq_mfma_rows(n_q * (n_q_heads / n_kv_heads)), v_bits, v_group)
                                : 0;
    const DecodeShape s = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, t_capacity, many_rows,
                                            rows_cap, vq_mfma);
    const Workspace w = make_workspace(cb->plan, s);
    // every entry point asks for the one documented size, whatever its own kernel needs (the static scratch
    // has been checked against the need of the kernels it serves)
    const size_t required = static_scratch_call ? w.total
                                                : std::max(w.total, octopus_attn_decode_workspace(cb, n_seq, n_q_heads, n_kv_heads,
                                                                                                  n_q, max_len));
    if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < required) return OCTOPUS_EWORKSPACE;
    char *base = static_cast<char *>(workspace);
    float *q_rot = reinterpret_cast<float *>(base + w.q_rot_off);
    float *part_ml = reinterpret_cast<float *>(base + w.part_ml_off);
    float *part_acc = reinterpret_cast<float *>(base + w.part_acc_off);
    float *q2 = with_qjl ? reinterpret_cast<float *>(base + w.q2_off) : nullptr;
    int32_t *work_plan = many_rows ? nullptr : reinterpret_cast<int32_t *>(base + w.plan_off);
    int err = launch_rotate_queries(cb->plan, q, q_dtype, signs, s, scale, q_rot, seq_lens, work_plan, signs2, q2,
                                    stream);
    if (err == 0 && ev_before != nullptr) err = record_event(ev_before, stream);
    if (err == 0) {
        if (with_qjl)
            err = launch_decode_qjl(*cb, s, q_rot, cache, qjl, q2, v, seq_lens, part_ml, part_acc, scores_out, work_plan,
                                    stream);
        else if (with_vq)
            err = launch_decode_vq(*cb, s, q_rot, cache, v, v_bits, v_group, seq_lens, part_ml, part_acc, scores_out,
                                   work_plan, stream);
        else
            err = launch_decode(*cb, s, q_rot, cache, v, v_dtype, seq_lens, part_ml, part_acc, scores_out, work_plan,
                                stream);
    }
    if (err == 0 && ev_after != nullptr) err = record_event(ev_after, stream);
    float *win_ml = nullptr, *win_acc = nullptr;
    if (err == 0 && win != nullptr) {
        win_ml = reinterpret_cast<float *>(base + w.win_ml_off);
        win_acc = reinterpret_cast<float *>(base + w.win_acc_off);
        err = launch_window(cb->plan, s, q, q_dtype, win->k_window, win->k_dtype, win->w_capacity, win->win_lens, v,
                            v_dtype, seq_lens, scale, win_ml, win_acc, scores_out, stream);
    }
    if (err == 0) err = launch_merge(cb->plan, s, part_ml, part_acc, work_plan, out, win_ml, win_acc, stream);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_attn_decode(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                        int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs, const void *cache,
                        int64_t t_capacity, const void *v, int32_t v_dtype, const int32_t *seq_lens,
                        int64_t max_len, float scale, float *out, float *scores_out, void *workspace,
                        size_t workspace_bytes, void *stream) {
    return attn_decode(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, cache, t_capacity, v, v_dtype,
                       seq_lens, max_len, scale, out, scores_out, workspace, workspace_bytes, stream, false, nullptr,
                       nullptr);
}

// ---- the entry point that allocates nothing ---------------------------------------------------------
// Scratch memory of octopus_attn_decode_static: a static device array, one copy per GPU for the life of the
// process.  Its name is only a host-side handle here: the device address is asked for once per device
// (hipGetSymbolAddress with that device current) and kept; kernels and everything else use that address.
static __device__ __align__(256) unsigned char scratch[OCTOPUS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, or NULL (with *err set) if the runtime refuses.
void *static_scratch(int *err) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *err = OCTOPUS_EHIP;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            *err = OCTOPUS_EHIP;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int octopus_attn_decode_static(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                               const void *cache, int64_t t_capacity, const void *v, int32_t v_dtype,
                               const int32_t *seq_lens, int64_t max_len, float scale, float *out, float *scores_out,
                               void *stream) {
    const int ok = decode_args_ok(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len);
    if (ok != OCTOPUS_OK) return ok;
    // the shapes must fit the static array: refused here, before anything is looked up or launched
    if (decode_args_ok(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len) != OCTOPUS_OK) return OCTOPUS_EINVAL;
    const size_t need = plain_decode_workspace(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len);
    if (need > static_cast<size_t>(OCTOPUS_STATIC_SCRATCH_BYTES)) return OCTOPUS_ESCRATCH;
    int err = OCTOPUS_OK;
    void *ws = static_scratch(&err);
    if (ws == nullptr) return err;
    // nothing in the scratch has to start at zero: the first kernel of the call writes the work plan and its
    // counter, and every partial result that the merge reads is written by the call's own main kernel
    return attn_decode(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, cache, t_capacity, v, v_dtype,
                       seq_lens, max_len, scale, out, scores_out, ws, OCTOPUS_STATIC_SCRATCH_BYTES, stream, false,
                       nullptr, nullptr, 0, 0, nullptr, true);
}

int octopus_attn_decode_hybrid(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                               const void *cache, int64_t t_capacity, const void *v, int32_t v_dtype,
                               const int32_t *seq_lens, int64_t max_len, const void *k_window, int32_t k_dtype,
                               int64_t w_capacity, const int32_t *win_lens, float scale, float *out, float *scores_out,
                               void *workspace, size_t workspace_bytes, void *stream) {
    WindowArgs win;
    win.k_window = k_window;
    win.k_dtype = k_dtype;
    win.w_capacity = w_capacity;
    win.win_lens = win_lens;
    return attn_decode(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, cache, t_capacity, v, v_dtype,
                       seq_lens, max_len, scale, out, scores_out, workspace, workspace_bytes, stream, false, nullptr,
                       nullptr, 0, 0, &win);
}

int octopus_attn_decode_qjl(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                            const uint8_t *signs2, const void *cache, const void *qjl, int64_t t_capacity,
                            const void *v, int32_t v_dtype, const int32_t *seq_lens, int64_t max_len, float scale,
                            float *out, float *scores_out, void *workspace, size_t workspace_bytes, void *stream) {
    return attn_decode(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, cache, t_capacity, v, v_dtype,
                       seq_lens, max_len, scale, out, scores_out, workspace, workspace_bytes, stream, true, signs2,
                       qjl);
}

static bool vq_params_ok(int32_t head_dim, int32_t bits, int32_t group) {
    return (head_dim == 64 || head_dim == 128 || head_dim == 256) && bits >= 2 && bits <= 4 &&
           (group == 16 || group == 32);
}

size_t octopus_vq_row_bytes(int32_t head_dim, int32_t bits, int32_t group) {
    if (!vq_params_ok(head_dim, bits, group)) return 0;
    return static_cast<size_t>(bits) * head_dim / 8 + static_cast<size_t>(head_dim / group) * 8;
}

size_t octopus_vq_bytes(int32_t head_dim, int32_t bits, int32_t group, int32_t n_seq, int32_t n_kv_heads,
                        int64_t t_capacity) {
    if (n_seq < 1 || n_kv_heads < 1 || t_capacity < 1) return 0;
    return octopus_vq_row_bytes(head_dim, bits, group) * n_seq * n_kv_heads * static_cast<size_t>(t_capacity);
}

static int encode_values(const void *v, int32_t v_dtype, int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                         int32_t n_seq, int32_t n_kv_heads, int32_t n_new, int32_t head_dim, int32_t bits,
                         int32_t group, void *vq, int64_t t_capacity, const int32_t *start_pos, void *stream,
                         PageTable pt) {
    if (v == nullptr || vq == nullptr) return OCTOPUS_EINVAL;
    if (n_seq < 1 || n_kv_heads < 1 || n_new < 0 || t_capacity < 1) return OCTOPUS_EINVAL;
    if (v_dtype != OCTOPUS_DTYPE_F32 && v_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
    if (!vq_params_ok(head_dim, bits, group)) return OCTOPUS_EUNSUPPORTED;
    if (stride_seq < 0 || stride_tok < 0 || stride_head < 0) return OCTOPUS_EINVAL;
    if (!aligned(v, 4) || !aligned(vq, 16)) return OCTOPUS_EINVAL;
    if (start_pos == nullptr && n_new > t_capacity) return OCTOPUS_EINVAL;
    if (static_cast<int64_t>(n_seq) * n_new * n_kv_heads * (head_dim / group) > (int64_t{1} << 38)) return OCTOPUS_EINVAL;
    // the launch: one sequence per grid z, a 32-bit index over the (token, KV head, group) triples of a slab of tokens
    if (n_seq > 65535 || static_cast<int64_t>(n_kv_heads) * (head_dim / group) > 4096) return OCTOPUS_EINVAL;
    if (n_new == 0) return OCTOPUS_OK;
    const int err = launch_encode_values(v, v_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new,
                                         head_dim, bits, group, vq, t_capacity, start_pos, stream, pt);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_encode_values(const void *v, int32_t v_dtype, int64_t stride_seq, int64_t stride_tok, int64_t stride_head,
                          int32_t n_seq, int32_t n_kv_heads, int32_t n_new, int32_t head_dim, int32_t bits,
                          int32_t group, void *vq, int64_t t_capacity, const int32_t *start_pos, void *stream) {
    return encode_values(v, v_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, head_dim, bits, group,
                         vq, t_capacity, start_pos, stream, PageTable{nullptr, 0, 0});
}

int octopus_attn_decode_vq(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                           int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs, const void *cache,
                           int64_t t_capacity, const void *vq, int32_t v_bits, int32_t v_group,
                           const int32_t *seq_lens, int64_t max_len, float scale, float *out, float *scores_out,
                           void *workspace, size_t workspace_bytes, void *stream) {
    if (v_bits == 0) return OCTOPUS_EUNSUPPORTED;
    return attn_decode(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, cache, t_capacity, vq,
                       OCTOPUS_DTYPE_F32, seq_lens, max_len, scale, out, scores_out, workspace, workspace_bytes, stream,
                       false, nullptr, nullptr, v_bits, v_group);
}

size_t octopus_paged_pool_bytes(const octopus_codebooks_t *cb, int32_t n_pages, int32_t n_kv_heads) {
    if (cb == nullptr || n_pages < 1 || n_kv_heads < 1 || !plan_consistent(cb->plan)) return 0;
    return static_cast<size_t>(n_pages) * n_kv_heads * OCTOPUS_TILE * cb->plan.granules * 16;
}

static bool page_table_ok(const void *pool, int32_t n_pages, const int32_t *block_table, int32_t max_pages_per_seq) {
    return pool != nullptr && block_table != nullptr && n_pages >= 1 && max_pages_per_seq >= 1 &&
           max_pages_per_seq <= (INT32_MAX / OCTOPUS_TILE) && aligned(pool, 16) && aligned(block_table, 4);
}

static int encode_paged(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                        int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                        const uint8_t *signs, void *k_pool, int32_t n_pages, const int32_t *block_table,
                        int32_t max_pages_per_seq, const int32_t *start_pos, void *stream, const uint8_t *signs2,
                        void *qjl_pool) {
    if (cb == nullptr || keys == nullptr || signs == nullptr) return OCTOPUS_EINVAL;
    if (qjl_pool != nullptr && !aligned(qjl_pool, 4)) return OCTOPUS_EINVAL;
    if (!page_table_ok(k_pool, n_pages, block_table, max_pages_per_seq)) return OCTOPUS_EINVAL;
    if (n_seq < 1 || n_kv_heads < 1 || n_new < 0) return OCTOPUS_EINVAL;
    if (n_seq > 65535 || n_kv_heads > 65535) return OCTOPUS_EINVAL;   // they are grid dimensions of the launch
    if (!plan_consistent(cb->plan)) return OCTOPUS_EINVAL;
    if (key_dtype != OCTOPUS_DTYPE_F32 && key_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
    if (!plan_supported(cb->plan) || !seed_grid_ok(*cb)) return OCTOPUS_EUNSUPPORTED;
    if (stride_seq < 0 || stride_tok < 0 || stride_head < 0) return OCTOPUS_EINVAL;
    if (stride_seq % 8 != 0 || stride_tok % 8 != 0 || stride_head % 8 != 0) return OCTOPUS_EINVAL;
    if (!aligned(keys, 16)) return OCTOPUS_EINVAL;
    const int64_t reach = static_cast<int64_t>(max_pages_per_seq) * OCTOPUS_TILE;   // tokens the table can address
    if (start_pos == nullptr && n_new > reach) return OCTOPUS_EINVAL;
    if (n_new == 0) return OCTOPUS_OK;
    const PageTable pt{block_table, max_pages_per_seq, n_pages};
    const int err = launch_encode_paged(*cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads,
                                        n_new, signs, k_pool, pt, start_pos, stream, signs2, qjl_pool);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_encode_paged(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                         int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                         const uint8_t *signs, void *k_pool, int32_t n_pages, const int32_t *block_table,
                         int32_t max_pages_per_seq, const int32_t *start_pos, void *stream) {
    return encode_paged(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, k_pool,
                        n_pages, block_table, max_pages_per_seq, start_pos, stream, nullptr, nullptr);
}

int octopus_encode_qjl_paged(const octopus_codebooks_t *cb, const void *keys, int32_t key_dtype, int64_t stride_seq,
                             int64_t stride_tok, int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new,
                             const uint8_t *signs, const uint8_t *signs2, void *k_pool, void *qjl_pool, int32_t n_pages,
                             const int32_t *block_table, int32_t max_pages_per_seq, const int32_t *start_pos,
                             void *stream) {
    if (signs2 == nullptr || qjl_pool == nullptr) return OCTOPUS_EINVAL;
    return encode_paged(cb, keys, key_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, signs, k_pool,
                        n_pages, block_table, max_pages_per_seq, start_pos, stream, signs2, qjl_pool);
}

static int attn_decode_paged(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                             int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                             const void *k_pool, const void *v_pool, int32_t n_pages, const int32_t *block_table,
                             int32_t max_pages_per_seq, const int32_t *seq_lens, int64_t max_len, float scale,
                             float *out, void *workspace, size_t workspace_bytes, void *stream, const WindowArgs *win,
                             int32_t v_bits = 0, int32_t v_group = 0, const uint8_t *signs2 = nullptr,
                             const void *qjl_pool = nullptr) {
    // v_bits > 0: v_pool holds group-quantised rows (the matrix-core kernel over them; no window)
    // qjl_pool: the QJL side-car in pages, scores corrected as in octopus_attn_decode_qjl (bf16 values, no window)
    const bool with_qjl = qjl_pool != nullptr;
    void *ev_before = g_event_before, *ev_after = g_event_after;
    g_event_before = g_event_after = nullptr;
    const int ok = decode_args_ok(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len);
    if (ok != OCTOPUS_OK) return ok;
    if (q == nullptr || signs == nullptr || seq_lens == nullptr || out == nullptr) return OCTOPUS_EINVAL;
    // A chunk of many query rows per KV head belongs to the many-row kernel (bf16 value pages, d <= 128, no QJL
    // side-car); where that does not serve, the call is refused rather than run as hundreds of row groups that
    // each read the keys again.
    const bool many_rows = many_rows_shape(cb->plan, n_q_heads, n_kv_heads, n_q) && v_bits == 0 && qjl_pool == nullptr;
    if (static_cast<int64_t>(n_q) * (n_q_heads / n_kv_heads) >= 32 && !many_rows) return OCTOPUS_EUNSUPPORTED;
    if (!plan_supported(cb->plan)) return OCTOPUS_EUNSUPPORTED;   // (a pair of the App. D sweep: no paged kernels)
    if (!page_table_ok(k_pool, n_pages, block_table, max_pages_per_seq) || v_pool == nullptr || !aligned(v_pool, 16))
        return OCTOPUS_EINVAL;
    const int64_t reach = static_cast<int64_t>(max_pages_per_seq) * OCTOPUS_TILE;
    if (max_len > reach) return OCTOPUS_EINVAL;
    if (q_dtype != OCTOPUS_DTYPE_F32 && q_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
    if (!aligned(q, 4) || !aligned(out, 4) || !std::isfinite(scale)) return OCTOPUS_EINVAL;
    if (win != nullptr) {
        if (win->k_window == nullptr || win->win_lens == nullptr || win->w_capacity < 1) return OCTOPUS_EINVAL;
        if (win->k_dtype != OCTOPUS_DTYPE_F32 && win->k_dtype != OCTOPUS_DTYPE_BF16) return OCTOPUS_EUNSUPPORTED;
        if (!aligned(win->k_window, 16)) return OCTOPUS_EINVAL;
    }
    if (with_qjl && (signs2 == nullptr || !aligned(qjl_pool, 4))) return OCTOPUS_EINVAL;
    const int rows_cap = with_qjl ? qjl_rows_cap(cb->plan) : 8;
    if (rows_cap <= 0) return OCTOPUS_EUNSUPPORTED;
    int32_t vq_waves = 0;
    if (v_bits != 0) {
        if (!vq_params_ok(cb->plan.head_dim, v_bits, v_group)) return OCTOPUS_EUNSUPPORTED;
        // over pages only the matrix-core kernel serves quantised values
        vq_waves = vq_mfma_available(cb->plan, vq_mfma_rows(n_q * (n_q_heads / n_kv_heads)), v_bits, v_group);
        if (vq_waves <= 0) return OCTOPUS_EUNSUPPORTED;
    }
    const DecodeShape s = make_decode_shape(cb->plan, n_seq, n_q_heads, n_kv_heads, n_q, max_len, reach, many_rows,
                                            rows_cap, vq_waves);
    const Workspace w = make_workspace(cb->plan, s);
    const size_t required = std::max(w.total, octopus_attn_decode_workspace(cb, n_seq, n_q_heads, n_kv_heads, n_q, max_len));
    if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < required) return OCTOPUS_EWORKSPACE;
    char *base = static_cast<char *>(workspace);
    float *q_rot = reinterpret_cast<float *>(base + w.q_rot_off);
    float *part_ml = reinterpret_cast<float *>(base + w.part_ml_off);
    float *part_acc = reinterpret_cast<float *>(base + w.part_acc_off);
    int32_t *work_plan = many_rows ? nullptr : reinterpret_cast<int32_t *>(base + w.plan_off);
    float *q2 = with_qjl ? reinterpret_cast<float *>(base + w.q2_off) : nullptr;
    const PageTable pt{block_table, max_pages_per_seq, n_pages};
    int err = launch_rotate_queries(cb->plan, q, q_dtype, signs, s, scale, q_rot, seq_lens, work_plan,
                                    with_qjl ? signs2 : nullptr, q2, stream);
    if (err == 0 && ev_before != nullptr) err = record_event(ev_before, stream);
    if (err == 0) {
        if (v_bits != 0)
            err = launch_decode_vq(*cb, s, q_rot, k_pool, v_pool, v_bits, v_group, seq_lens, part_ml, part_acc, nullptr,
                                   work_plan, stream, pt);
        else if (with_qjl)
            err = launch_decode_paged_qjl(*cb, s, q_rot, k_pool, qjl_pool, q2, v_pool, pt, seq_lens, part_ml, part_acc,
                                          work_plan, stream);
        else
            err = launch_decode_paged(*cb, s, q_rot, k_pool, v_pool, pt, seq_lens, part_ml, part_acc, work_plan, stream);
    }
    if (err == 0 && ev_after != nullptr) err = record_event(ev_after, stream);
    float *win_ml = nullptr, *win_acc = nullptr;
    if (err == 0 && win != nullptr) {
        // the window's value rows follow the compressed tokens in the sequence's pages
        win_ml = reinterpret_cast<float *>(base + w.win_ml_off);
        win_acc = reinterpret_cast<float *>(base + w.win_acc_off);
        err = launch_window(cb->plan, s, q, q_dtype, win->k_window, win->k_dtype, win->w_capacity, win->win_lens, v_pool,
                            OCTOPUS_DTYPE_BF16, seq_lens, scale, win_ml, win_acc, nullptr, stream, pt);
    }
    if (err == 0) err = launch_merge(cb->plan, s, part_ml, part_acc, work_plan, out, win_ml, win_acc, stream);
    return err == 0 ? OCTOPUS_OK : OCTOPUS_EHIP;
}

int octopus_attn_decode_paged(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                              const void *k_pool, const void *v_pool, int32_t n_pages, const int32_t *block_table,
                              int32_t max_pages_per_seq, const int32_t *seq_lens, int64_t max_len, float scale,
                              float *out, void *workspace, size_t workspace_bytes, void *stream) {
    return attn_decode_paged(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, k_pool, v_pool, n_pages,
                             block_table, max_pages_per_seq, seq_lens, max_len, scale, out, workspace, workspace_bytes,
                             stream, nullptr);
}

int octopus_attn_decode_paged_hybrid(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                                     int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                                     const void *k_pool, const void *v_pool, int32_t n_pages,
                                     const int32_t *block_table, int32_t max_pages_per_seq, const int32_t *seq_lens,
                                     int64_t max_len, const void *k_window, int32_t k_dtype, int64_t w_capacity,
                                     const int32_t *win_lens, float scale, float *out, void *workspace,
                                     size_t workspace_bytes, void *stream) {
    WindowArgs win;
    win.k_window = k_window;
    win.k_dtype = k_dtype;
    win.w_capacity = w_capacity;
    win.win_lens = win_lens;
    return attn_decode_paged(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, k_pool, v_pool, n_pages,
                             block_table, max_pages_per_seq, seq_lens, max_len, scale, out, workspace, workspace_bytes,
                             stream, &win);
}

int octopus_encode_values_paged(const void *v, int32_t v_dtype, int64_t stride_seq, int64_t stride_tok,
                                int64_t stride_head, int32_t n_seq, int32_t n_kv_heads, int32_t n_new, int32_t head_dim,
                                int32_t bits, int32_t group, void *vq_pool, int32_t n_pages, const int32_t *block_table,
                                int32_t max_pages_per_seq, const int32_t *start_pos, void *stream) {
    if (!page_table_ok(vq_pool, n_pages, block_table, max_pages_per_seq)) return OCTOPUS_EINVAL;
    // the table addresses max_pages_per_seq * 64 tokens per sequence: that is the capacity rows are dropped beyond
    const int64_t reach = static_cast<int64_t>(max_pages_per_seq) * OCTOPUS_TILE;
    return encode_values(v, v_dtype, stride_seq, stride_tok, stride_head, n_seq, n_kv_heads, n_new, head_dim, bits, group,
                         vq_pool, reach, start_pos, stream, PageTable{block_table, max_pages_per_seq, n_pages});
}

int octopus_attn_decode_paged_vq(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                                 const void *k_pool, const void *vq_pool, int32_t v_bits, int32_t v_group,
                                 int32_t n_pages, const int32_t *block_table, int32_t max_pages_per_seq,
                                 const int32_t *seq_lens, int64_t max_len, float scale, float *out, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    if (v_bits == 0) return OCTOPUS_EUNSUPPORTED;
    return attn_decode_paged(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, k_pool, vq_pool, n_pages,
                             block_table, max_pages_per_seq, seq_lens, max_len, scale, out, workspace, workspace_bytes,
                             stream, nullptr, v_bits, v_group);
}

int octopus_attn_decode_paged_qjl(const octopus_codebooks_t *cb, const void *q, int32_t q_dtype, int32_t n_seq,
                                  int32_t n_q_heads, int32_t n_kv_heads, int32_t n_q, const uint8_t *signs,
                                  const uint8_t *signs2, const void *k_pool, const void *qjl_pool, const void *v_pool,
                                  int32_t n_pages, const int32_t *block_table, int32_t max_pages_per_seq,
                                  const int32_t *seq_lens, int64_t max_len, float scale, float *out, void *workspace,
                                  size_t workspace_bytes, void *stream) {
    if (signs2 == nullptr || qjl_pool == nullptr) return OCTOPUS_EINVAL;
    return attn_decode_paged(cb, q, q_dtype, n_seq, n_q_heads, n_kv_heads, n_q, signs, k_pool, v_pool, n_pages,
                             block_table, max_pages_per_seq, seq_lens, max_len, scale, out, workspace, workspace_bytes,
                             stream, nullptr, 0, 0, signs2, qjl_pool);
}

const char *octopus_strerror(int code) {
    switch (code) {
        case OCTOPUS_OK: return "ok";
        case OCTOPUS_EINVAL: return "invalid argument";
        case OCTOPUS_EUNSUPPORTED: return "unsupported head_dim, bit width, dtype or head ratio";
        case OCTOPUS_EWORKSPACE: return "workspace missing, misaligned or too small";
        case OCTOPUS_EHIP: return "HIP launch failed";
        case OCTOPUS_ESCRATCH:
            return "shapes need more scratch memory than the library's static array holds (OCTOPUS_STATIC_SCRATCH_BYTES)";
        default: return "unknown error";
    }
}

}  // extern "C"
