// Host side of the library (plans, codebooks, argument checks, workspace carve-up, dispatch) under the host
// sanitizers, without a GPU: the kernel launchers are replaced by stubs that check nothing and launch nothing.
// Built by tests/test_sanitizers.py from this file plus csrc/octopus_host.cpp.
#include <cstdio>
#include <cstring>
#include <vector>

#include "octopus_internal.h"

namespace octopus {
int g_launches = 0;
int launch_rotate_queries(const octopus_plan_t &, const void *, int, const uint8_t *, const DecodeShape &, float, float *,
                          const int32_t *, int32_t *, const uint8_t *, float *, void *) { ++g_launches; return 0; }
int launch_decode(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *, int,
                  const int32_t *, float *, float *, float *, int32_t *, void *) { ++g_launches; return 0; }
int launch_decode_qjl(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *,
                      const float *, const void *, const int32_t *, float *, float *, float *, int32_t *, void *) { ++g_launches; return 0; }
int qjl_rows_cap(const octopus_plan_t &) { return 4; }
int launch_merge(const octopus_plan_t &, const DecodeShape &, const float *, const float *, const int32_t *, float *,
                 const float *, const float *, void *) { ++g_launches; return 0; }
int launch_window(const octopus_plan_t &, const DecodeShape &, const void *, int, const void *, int, int64_t,
                  const int32_t *, const void *, int, const int32_t *, float, float *, float *, float *, void *, PageTable) { ++g_launches; return 0; }
int launch_encode(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t, int32_t, int32_t, int32_t,
                  const uint8_t *, void *, int64_t, const int32_t *, const uint8_t *, void *, void *) { ++g_launches; return 0; }
int launch_encode_paged(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t, int32_t, int32_t,
                        int32_t, const uint8_t *, void *, const PageTable &, const int32_t *, void *, const uint8_t *, void *) { ++g_launches; return 0; }
int launch_decode_paged_qjl(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *,
                            const float *, const void *, const PageTable &, const int32_t *, float *, float *, int32_t *, void *) { ++g_launches; return 0; }
int launch_decode_paged(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *,
                        const PageTable &, const int32_t *, float *, float *, int32_t *, void *) { ++g_launches; return 0; }
int launch_encode_rounding(const octopus_codebooks_t &, const void *, int, int64_t, int64_t, int64_t, int32_t, int32_t,
                           int32_t, const uint8_t *, void *, int64_t, const int32_t *, int32_t, void *) { ++g_launches; return 0; }
int launch_encode_values(const void *, int, int64_t, int64_t, int64_t, int32_t, int32_t, int32_t, int32_t, int32_t,
                         int32_t, void *, int64_t, const int32_t *, void *, PageTable) { ++g_launches; return 0; }
int launch_decode_vq(const octopus_codebooks_t &, const DecodeShape &, const float *, const void *, const void *, int,
                     int, const int32_t *, float *, float *, float *, int32_t *, void *, PageTable) { ++g_launches; return 0; }
int record_event(void *, void *) { return 0; }
int launch_probe_read(const void *, int64_t, int, int, void *, void *) { ++g_launches; return 0; }
bool plan_supported(const octopus_plan_t &p) { return p.b_dir[0] <= 5 && p.b_nrm[0] <= 3; }
bool plan_sweep_only(const octopus_plan_t &p) { return p.head_dim == 128 && !plan_supported(p); }
int vq_mfma_available(const octopus_plan_t &p, int32_t, int32_t v_bits, int32_t v_group) { return plan_supported(p) && v_bits == 3 && v_group == 32 ? (p.head_dim <= 128 ? 8 : 4) : 0; }
}  // namespace octopus

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main() {
    const float widths[] = {1.0f, 1.5f, 2.0f, 2.5f, 3.0f, 4.0f};
    const int dims[] = {64, 128, 256};
    // addresses that satisfy the alignment checks; the stubs never look behind them
    alignas(256) static unsigned char fake[4096];
    void *p = fake;
    for (int d : dims)
        for (float b : widths) {
            octopus_codebooks_t cb;
            EXPECT(octopus_build_codebooks(d, b, &cb) == OCTOPUS_OK);
            EXPECT(cb.plan.n_tri == (d + 2) / 3 && cb.plan.record_bytes == 4 + cb.plan.dir_bytes + cb.plan.nrm_bytes);
            for (int c = 0; c < cb.plan.n_class; ++c)
                for (int k = 0; k + 1 < (1 << cb.plan.b_dir[c]); ++k) EXPECT(cb.c_xi[c][k] < cb.c_xi[c][k + 1]);
            EXPECT(octopus_cache_bytes(&cb, 2, 3, 128) == size_t(2) * 3 * 128 * cb.plan.granules * 16);
            EXPECT(octopus_cache_bytes(&cb, 2, 3, 100) == 0);
            const size_t ws = octopus_attn_decode_workspace(&cb, 3, 8, 2, 1, 1000);
            EXPECT(ws > 0 && ws % 256 == 0);
            EXPECT(octopus_attn_decode_workspace(&cb, 3, 8, 3, 1, 1000) == 0);   // heads not divisible
            EXPECT(octopus_qjl_bytes(&cb, 1, 1, 64) == size_t(64) * (d / 8 + 2));
            EXPECT(octopus_paged_pool_bytes(&cb, 5, 2) == size_t(5) * 2 * 64 * cb.plan.granules * 16);
            // calls that pass validation reach the (stubbed) launchers
            const int before = octopus::g_launches;
            EXPECT(octopus_encode(&cb, p, OCTOPUS_DTYPE_BF16, 8 * d, d, d, 1, 1, 8, fake, p, 64, nullptr, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_encode(&cb, p, OCTOPUS_DTYPE_BF16, 8 * d, d, d, 1, 1, 0, fake, p, 64, nullptr, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_encode(&cb, nullptr, OCTOPUS_DTYPE_BF16, 8 * d, d, d, 1, 1, 8, fake, p, 64, nullptr, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_encode(&cb, p, 7, 8 * d, d, d, 1, 1, 8, fake, p, 64, nullptr, nullptr) == OCTOPUS_EUNSUPPORTED);
            EXPECT(octopus_encode(&cb, p, OCTOPUS_DTYPE_BF16, 8 * d, d + 1, d, 1, 1, 8, fake, p, 64, nullptr, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_encode_rounding(&cb, p, OCTOPUS_DTYPE_F32, 8 * d, d, d, 1, 1, 8, fake, p, 64, nullptr, 9, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_encode_rounding(&cb, p, OCTOPUS_DTYPE_F32, 8 * d, d, d, 1, 1, 8, fake, p, 64, nullptr, OCTOPUS_ROUND_FULL, nullptr) == OCTOPUS_OK);
            std::vector<unsigned char> wsbuf(ws + 512);
            void *wsp = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(wsbuf.data()) + 255) & ~uintptr_t(255));
            EXPECT(octopus_attn_decode(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1024, p, OCTOPUS_DTYPE_BF16,
                                       reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                       nullptr, wsp, ws, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_attn_decode(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1024, p, OCTOPUS_DTYPE_BF16,
                                       reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                       nullptr, wsp, ws - 1, nullptr) == OCTOPUS_EWORKSPACE);
            EXPECT(octopus_attn_decode(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1000, p, OCTOPUS_DTYPE_BF16,
                                       reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                       nullptr, wsp, ws, nullptr) == OCTOPUS_EINVAL);    // capacity not a multiple of 64
            EXPECT(octopus_attn_decode_hybrid(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1024, p, OCTOPUS_DTYPE_BF16,
                                              reinterpret_cast<const int32_t *>(fake), 1000, nullptr, OCTOPUS_DTYPE_BF16, 32,
                                              reinterpret_cast<const int32_t *>(fake), 0.1f, reinterpret_cast<float *>(fake),
                                              nullptr, wsp, ws, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_attn_decode_vq(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1024, p, 5, 32,
                                          reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                          nullptr, wsp, ws, nullptr) == OCTOPUS_EUNSUPPORTED);
            int32_t table[64] = {0};
            EXPECT(octopus_attn_decode_paged(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 40, table, 16,
                                             reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                             wsp, ws, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_attn_decode_paged(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 40, table, 15,
                                             reinterpret_cast<const int32_t *>(fake), 1000, 0.1f, reinterpret_cast<float *>(fake),
                                             wsp, ws, nullptr) == OCTOPUS_EINVAL);      // the table cannot hold max_len
            // the paged forms of the variants: window, quantised values (3 bits, groups of 32: the stub's one build),
            // the QJL side-car, a chunk of 40 query rows per KV head (the many-row kernel, up to head_dim 128)
            const int32_t *ip = reinterpret_cast<const int32_t *>(fake);
            float *fp = reinterpret_cast<float *>(fake);
            EXPECT(octopus_attn_decode_paged_hybrid(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 40, table, 16, ip, 1000,
                                                    p, OCTOPUS_DTYPE_BF16, 32, ip, 0.1f, fp, wsp, ws, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_attn_decode_paged_hybrid(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 40, table, 16, ip, 1000,
                                                    p, OCTOPUS_DTYPE_BF16, 0, ip, 0.1f, fp, wsp, ws, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_attn_decode_paged_vq(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 3, 32, 40, table, 16, ip, 1000,
                                                0.1f, fp, wsp, ws, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_attn_decode_paged_vq(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, p, 3, 16, 40, table, 16, ip, 1000,
                                                0.1f, fp, wsp, ws, nullptr) == OCTOPUS_EUNSUPPORTED);   // (no such build in the stub)
            EXPECT(octopus_attn_decode_paged_qjl(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, fake, p, p, p, 40, table, 16, ip,
                                                 1000, 0.1f, fp, wsp, ws, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_attn_decode_paged_qjl(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, nullptr, p, p, p, 40, table, 16, ip,
                                                 1000, 0.1f, fp, wsp, ws, nullptr) == OCTOPUS_EINVAL);
            EXPECT(octopus_encode_qjl_paged(&cb, p, OCTOPUS_DTYPE_BF16, 8 * d, d, d, 1, 1, 8, fake, fake, p, p, 40, table, 16,
                                            nullptr, nullptr) == OCTOPUS_OK);
            EXPECT(octopus_encode_values_paged(p, OCTOPUS_DTYPE_BF16, 8 * d, d, d, 1, 1, 8, d, 3, 32, p, 40, table, 16, nullptr,
                                               nullptr) == OCTOPUS_OK);
            {
                const size_t ws40 = octopus_attn_decode_workspace(&cb, 1, 8, 2, 10, 1000);
                std::vector<unsigned char> buf40(ws40 + 512);
                void *w40 = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(buf40.data()) + 255) & ~uintptr_t(255));
                EXPECT(octopus_attn_decode_paged(&cb, p, OCTOPUS_DTYPE_BF16, 1, 8, 2, 10, fake, p, p, 40, table, 16, ip, 1000, 0.1f,
                                                 fp, w40, ws40, nullptr) == (d <= 128 ? OCTOPUS_OK : OCTOPUS_EUNSUPPORTED));
                EXPECT(octopus_attn_decode_paged_vq(&cb, p, OCTOPUS_DTYPE_BF16, 1, 8, 2, 10, fake, p, p, 3, 32, 40, table, 16, ip,
                                                    1000, 0.1f, fp, w40, ws40, nullptr) == OCTOPUS_EUNSUPPORTED);
            }
            EXPECT(octopus::g_launches > before);
            // the entry point on the static scratch: refused before any runtime call when the shapes exceed it;
            // otherwise it needs a device for the array's address and reports the runtime's refusal
            const int rc = octopus_attn_decode_static(&cb, p, OCTOPUS_DTYPE_BF16, 3, 8, 2, 1, fake, p, 1024, p,
                                                      OCTOPUS_DTYPE_BF16, reinterpret_cast<const int32_t *>(fake), 1000, 0.1f,
                                                      reinterpret_cast<float *>(fake), nullptr, nullptr);
            EXPECT(rc == OCTOPUS_OK || rc == OCTOPUS_EHIP);
        }
    octopus_codebooks_t cb;
    EXPECT(octopus_build_codebooks(128, 3.5f, &cb) == OCTOPUS_EUNSUPPORTED);
    EXPECT(octopus_build_codebooks(96, 3.0f, &cb) == OCTOPUS_EUNSUPPORTED);
    EXPECT(octopus_build_codebooks(128, 3.0f, nullptr) == OCTOPUS_EINVAL);
    EXPECT(octopus_build_codebooks_pair(128, 3, 3, &cb) == OCTOPUS_OK);
    EXPECT(octopus_build_codebooks_pair(128, 0, 3, &cb) == OCTOPUS_EUNSUPPORTED);
    EXPECT(octopus_build_codebooks_pair(128, 6, 6, &cb) == OCTOPUS_OK && cb.plan.record_bytes == 4 + 66 + 33);
    EXPECT(octopus_build_codebooks_pair(128, 7, 2, &cb) == OCTOPUS_EUNSUPPORTED);
    EXPECT(octopus_vq_row_bytes(128, 3, 32) == 80 && octopus_vq_row_bytes(128, 5, 32) == 0);
    EXPECT(octopus_encode_values(fake, OCTOPUS_DTYPE_BF16, 1024, 128, 128, 1, 1, 4, 128, 3, 32, fake, 64, nullptr, nullptr) == OCTOPUS_OK);
    EXPECT(octopus_profile_events(fake, nullptr) == OCTOPUS_EINVAL);
    EXPECT(octopus_probe_read(fake, 4096, 1, 4, fake, nullptr) == OCTOPUS_OK);
    EXPECT(octopus_probe_read(fake, 16, 1, 4, fake, nullptr) == OCTOPUS_EINVAL);
    for (int code = 1; code >= -6; --code) EXPECT(std::strlen(octopus_strerror(code)) > 0);
    // a video-chunk shape needs more scratch than the static array holds
    EXPECT(octopus_build_codebooks(64, 4.0f, &cb) == OCTOPUS_OK);
    EXPECT(octopus_attn_decode_workspace(&cb, 1, 24, 24, 3600, 75648) > size_t(OCTOPUS_STATIC_SCRATCH_BYTES));
    EXPECT(octopus_attn_decode_static(&cb, p, OCTOPUS_DTYPE_BF16, 1, 24, 24, 3600, fake, p, 75648, p, OCTOPUS_DTYPE_BF16,
                                      reinterpret_cast<const int32_t *>(fake), 75600, 0.1f, reinterpret_cast<float *>(fake),
                                      nullptr, nullptr) == OCTOPUS_ESCRATCH);
    std::printf(failures ? "FAILED (%d)\n" : "host driver ok\n", failures);
    return failures ? 1 : 0;
}
