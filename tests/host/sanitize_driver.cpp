// Host-side driver for the sanitizer build of the library (AddressSanitizer + UndefinedBehaviorSanitizer
// on the host code; needs no GPU): walks the argument validation, workspace arithmetic and host-only
// functions of every entry point of include/sp.h with valid, invalid and extreme host-visible
// arguments. Device pointers are fake and never dereferenced: every call must return before a launch.
#include "sp.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static int g_fail = 0;
#define EXPECT(cond)                                                             \
    do {                                                                         \
        if (!(cond)) { std::printf("FAILED %s:%d: %s (last error: %s)\n", __FILE__, __LINE__, #cond, sp_last_error()); ++g_fail; } \
    } while (0)

int main()
{
    void *fake = reinterpret_cast<void *>(0x10000);
    // ---- host-only arithmetic ----
    EXPECT(sp_keep_count(2048, 10, 100) == 205);
    EXPECT(sp_keep_count(INT64_MAX, INT64_MAX, 1) == INT64_MAX);
    EXPECT(sp_keep_count(INT64_MAX, 1, INT64_MAX) == 1);
    EXPECT(sp_keep_count(0, 1, 2) == -1);
    EXPECT(std::strstr(sp_version(), "gfx950") != nullptr);

    // ---- score descriptors and workspaces over a sweep of shapes and sizes ----
    const int dims[] = {64, 128, 96};
    for (int d : dims)
        for (int layers : {1, 16, 128, 129})
            for (int kv : {1, 8, 512})
                for (int g : {1, 4, 16, 17})
                    for (int nq : {1, 8, 16, 17}) {
                        sp_score_desc desc{layers, kv * g, kv, d, nq, 0.125f, SP_LAYER_MEAN, (int64_t)d, (int64_t)d * 4096};
                        for (int64_t tokens : {(int64_t)0, (int64_t)1, (int64_t)513, (int64_t)131072, (int64_t)1 << 40}) {
                            size_t n = 0;
                            const sp_status rc = sp_score_workspace(&desc, tokens, 1, &n);
                            EXPECT(rc == SP_OK || rc == SP_ERR_UNSUPPORTED || rc == SP_ERR_INVALID_ARG);
                            if (rc == SP_OK) EXPECT(n % 256 == 0);
                            (void)sp_score_is_fused(&desc, tokens);
                        }
                        size_t n = 0;
                        (void)sp_score_workspace(&desc, 100000, 4096, &n);
                        EXPECT(sp_score_workspace(&desc, 100000, 4097, &n) != SP_OK);
                    }
    sp_score_desc ok{2, 4, 2, 64, 8, 0.125f, SP_LAYER_MEAN, 64, 64 * 1024};
    size_t wsn = 0;
    EXPECT(sp_score_workspace(&ok, 1024, 1, &wsn) == SP_OK && wsn > 0);
    EXPECT(sp_score_workspace(nullptr, 1024, 1, &wsn) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_workspace(&ok, 1024, 1, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_workspace(&ok, -1, 1, &wsn) == SP_ERR_INVALID_ARG);
    const void *layers[2] = {fake, fake};
    const void *bad_layers[2] = {fake, nullptr};
    const void *odd_layers[2] = {fake, reinterpret_cast<void *>(0x10008)};
    float *scores = static_cast<float *>(fake);
    EXPECT(sp_score(&ok, nullptr, layers, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score(&ok, fake, nullptr, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score(&ok, fake, bad_layers, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score(&ok, fake, odd_layers, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score(&ok, fake, layers, -5, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score(&ok, fake, layers, 0, scores, fake, wsn, nullptr) == SP_OK);         // nothing to do
    EXPECT(sp_score(&ok, fake, layers, 1024, scores, nullptr, 0, nullptr) == SP_ERR_WORKSPACE);
    EXPECT(sp_score(&ok, fake, layers, 1024, scores, fake, 256, nullptr) == SP_ERR_WORKSPACE);
    EXPECT(sp_score(&ok, fake, layers, 1024, scores, reinterpret_cast<void *>(0x10010), wsn, nullptr) == SP_ERR_WORKSPACE);
    EXPECT(sp_score_look(&ok, fake, layers, 1024, nullptr, 0, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_look(&ok, fake, layers, 1024, fake, 2, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_paged(&ok, fake, layers, nullptr, 4096, 8192, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_paged(&ok, fake, layers, static_cast<const int32_t *>(fake), 100, 8192, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);
    EXPECT(sp_score_fp8(&ok, fake, layers, nullptr, 1024, scores, fake, wsn, nullptr) == SP_ERR_INVALID_ARG);

    // ---- ragged batches: offsets of every kind ----
    {
        std::vector<int64_t> off = {0, 300, 301, 301, 814, 1070, 1147};
        size_t bn = 0;
        EXPECT(sp_score_workspace(&ok, off.back(), 6, &bn) == SP_OK);
        EXPECT(sp_score_batch(&ok, fake, layers, nullptr, static_cast<const int64_t *>(fake), 6, scores, fake, bn, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_score_batch(&ok, fake, layers, off.data(), nullptr, 6, scores, fake, bn, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_score_batch(&ok, fake, layers, off.data(), static_cast<const int64_t *>(fake), 0, scores, fake, bn, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_score_batch(&ok, fake, layers, off.data(), static_cast<const int64_t *>(fake), 6, scores, fake, 256, nullptr) == SP_ERR_WORKSPACE);
        std::vector<int64_t> dec = {0, 300, 200};
        EXPECT(sp_score_batch(&ok, fake, layers, dec.data(), static_cast<const int64_t *>(fake), 2, scores, fake, bn, nullptr) == SP_ERR_INVALID_ARG);
        std::vector<int64_t> nz = {5, 300};
        EXPECT(sp_score_batch(&ok, fake, layers, nz.data(), static_cast<const int64_t *>(fake), 1, scores, fake, bn, nullptr) == SP_ERR_INVALID_ARG);
        std::vector<int64_t> empty(4097, 0);
        EXPECT(sp_score_batch(&ok, fake, layers, empty.data(), static_cast<const int64_t *>(fake), 4096, scores, fake, bn, nullptr) == SP_OK);
        EXPECT(sp_score_batch_is_fused(&ok, off.data(), 6) == 0);
        EXPECT(sp_score_batch_is_fused(&ok, dec.data(), 2) == -1);
        std::vector<int64_t> big(4097);
        for (int i = 0; i <= 4096; ++i) big[i] = (int64_t)i * 70000;
        EXPECT(sp_score_batch_is_fused(&ok, big.data(), 4096) >= 0);
    }

    // ---- selection ----
    {
        size_t n = 0;
        EXPECT(sp_select_workspace(1000, 32, &n) == SP_OK && n >= 32 * 4);
        EXPECT(sp_select_workspace(0, 32, &n) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select_workspace(INT64_MAX / 2, 1, &n) == SP_OK);
        int32_t *sel = static_cast<int32_t *>(fake);
        int64_t *spans = static_cast<int64_t *>(fake);
        EXPECT(sp_select(scores, 1000, 13, 32, 4, sel, spans, sel, nullptr, fake, 0, nullptr) == SP_ERR_WORKSPACE);
        EXPECT(sp_select(scores, 1000, 12, 32, 4, sel, spans, sel, nullptr, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select(scores, 1000, 131, 32, 4, sel, spans, sel, nullptr, fake, n, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select(scores, 1000, 13, 32, 33, sel, spans, sel, nullptr, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select(scores, INT64_MAX, 13, 1, 4, sel, spans, sel, nullptr, fake, n, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select_static(scores, (1 << 18) + 1, 1, 1, 1, sel, spans, sel, nullptr, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select_static(nullptr, 1000, 13, 32, 4, sel, spans, sel, nullptr, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select_budget_workspace(4096, 32, &n) == SP_OK);
        EXPECT(sp_select_budget_workspace((int64_t)1 << 22, 32, &n) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select_budget(scores, 4096, 13, 32, spans, spans, 5000, -1, sel, spans, sel, spans, nullptr, nullptr, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select_budget(scores, 4096, 13, 32, spans, spans, (int64_t)1 << 31, 10, sel, spans, sel, spans, nullptr, nullptr, fake, n, nullptr) == SP_ERR_UNSUPPORTED);
    }

    // ---- projection, assembly, probe ----
    {
        int64_t *p64 = static_cast<int64_t *>(fake);
        int32_t *p32 = static_cast<int32_t *>(fake);
        EXPECT(sp_project(nullptr, 10, p64, 12, p64, p32, 4, p64, p32, nullptr, p64, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_project(p64, 0, p64, 12, p64, p32, 4, p64, p32, nullptr, p64, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_project(p64, 10, p64, 12, p64, p32, (1 << 24) + 1, p64, p32, nullptr, p64, nullptr) == SP_ERR_INVALID_ARG);
        size_t n = 0;
        EXPECT(sp_assemble_workspace(100, &n) == SP_OK && n > 0);
        EXPECT(sp_assemble_workspace(0, &n) == SP_ERR_INVALID_ARG);
        EXPECT(sp_assemble(p32, 100, p64, p32, 10, nullptr, 3, 50, p32, p32, nullptr, p64, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_assemble(p32, 100, p64, p32, 10, p32, 2000, 50, p32, p32, nullptr, p64, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        // ragged-batch select / project: host arrays are walked before anything else happens
        const int64_t off[4] = {0, 400, 400, 1000}, moff[4] = {0, 450, 450, 1100}, kept[4] = {0, 3, 3, 7};
        const int64_t bad_kept[4] = {0, 14, 14, 18}, huge_off[2] = {0, INT64_MAX}, many[2] = {0, 1025}, one[2] = {0, 1};
        float *scores = static_cast<float *>(fake);
        EXPECT(sp_select_batch_workspace(1000, 3, 32, &n) == SP_OK && n % 256 == 0);
        EXPECT(sp_select_batch_workspace(INT64_MAX, 4096, 1, &n) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select_batch(scores, off, p64, 3, 13, 32, bad_kept, p64, p32, p64, p32, nullptr, fake, n, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_select_batch(scores, huge_off, p64, 1, 13, 1, one, p64, p32, p64, p32, nullptr, fake, n, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_select_batch(scores, off, p64, 3, 13, 32, kept, p64, p32, p64, p32, nullptr, fake, 8, nullptr) == SP_ERR_WORKSPACE);
        EXPECT(sp_project_batch(p64, off, p64, p64, moff, p64, 3, p64, p32, bad_kept, nullptr, p64, p32, nullptr, p64, nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_project_batch(p64, huge_off, p64, p64, huge_off, p64, 1, p64, p32, one, p64, p64, p32, nullptr, p64, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_project_batch(p64, off, p64, p64, moff, p64, 1, p64, p32, many, p64, p64, p32, nullptr, p64, nullptr) == SP_ERR_UNSUPPORTED);
        EXPECT(sp_hbm_read_probe(nullptr, 1024, static_cast<uint64_t *>(fake), nullptr) == SP_ERR_INVALID_ARG);
        EXPECT(sp_hbm_read_probe(fake, 24, static_cast<uint64_t *>(fake), nullptr) == SP_ERR_INVALID_ARG);
    }
    sp_debug_fused_giveup(4, 1);
    sp_debug_fused_giveup(1u << 20, 0);
    std::printf(g_fail ? "sanitize driver: %d check(s) failed\n" : "sanitize driver: all checks passed\n", g_fail);
    return g_fail ? 1 : 0;
}
