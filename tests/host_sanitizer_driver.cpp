// Host-side paths of libsconv exercised under AddressSanitizer + UndefinedBehaviorSanitizer (built and run by
// tests/test_host_sanitizers.py from host-only objects: no device code, no GPU).  Every call here must return
// before anything is launched; the sanitizers watch the argument checks, size arithmetic, naming and planning
// code on the way.  Prints "ok" and exits 0 when every expectation holds.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <initializer_list>

#include "sconv.h"

static int failures = 0;
#define EXPECT(cond)                                                       \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "line %d: %s does not hold\n", __LINE__, #cond); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

static sconv_desc_t desc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int groups,
                         int ph = 0, int pw = 0, int ps = 0, int flags = 0)
{
    sconv_desc_t d = {N, C, H, W, K, R, S, stride, pad, groups, ph, pw, ps, flags};
    return d;
}

int main()
{
    int32_t oh = 0, ow = 0, ph = 0, pw = 0;
    int64_t rows = 0, slots = 0;
    size_t bytes = 0;
    char name[64];
    void* fake = reinterpret_cast<void*>(uintptr_t(256));   // never dereferenced: every call below fails earlier
    float* ffake = static_cast<float*>(fake);

    // sizes
    sconv_desc_t d = desc(2, 16, 28, 28, 32, 3, 3, 1, 1, 1, 2, 2, 2, SCONV_RELU);
    EXPECT(sconv_output_dims(&d, &oh, &ow, &ph, &pw) == SCONV_OK && oh == 28 && ow == 28 && ph == 14 && pw == 14);
    EXPECT(sconv_output_dims(&d, &oh, &ow, nullptr, nullptr) == SCONV_OK);
    EXPECT(sconv_encode_sizes(&d, SCONV_FMT_ECR, &rows, &slots) == SCONV_OK && rows == 2 * 784 && slots == 144);
    EXPECT(sconv_encode_sizes(&d, SCONV_FMT_PECR, &rows, &slots) == SCONV_OK && rows == 2 * 14 * 14 * 4);
    EXPECT(sconv_encode_sizes(&d, 7, &rows, &slots) == SCONV_EINVAL);
    EXPECT(sconv_output_dims(nullptr, &oh, &ow, nullptr, nullptr) == SCONV_EINVAL);

    // descriptors at the edge of the integer ranges: no overflow on the way to the verdict
    const int big = 0x7fffffff;
    sconv_desc_t edge[] = {
        desc(1, 16, 8, 8, 32, big, big, 1, 1 << 30, 1),  desc(1, 16, big, big, 32, 3, 3, 1, 1, 1),
        desc(big, big, big, big, big, 3, 3, 1, 1, 1),     desc(1, 16, 8, 8, 32, 3, 3, big, 1, 1),
        desc(1, big, 1, 1, big, 1, 1, 1, 0, big),         desc(1, 16, 8, 8, 32, 3, 3, 1, 1, 1, big, big, big),
        desc(1, 16, 8, 8, 32, 3, 3, 1, 1, 1, 2, 2, big),  desc(1, 16, big, 8, 32, 3, 3, 1, 2, 1, 2, 2, 1),
        desc(-big, 16, 8, 8, 32, 3, 3, 1, 1, 1),          desc(1, 16, 8, 8, 32, 3, 3, 1, -big, 1),
        desc(1 << 20, 1 << 10, 1, 1, 1 << 10, 1, 1, 1, 0, 1), desc(1, 1 << 22, 4, 4, 8, 3, 3, 1, 1, 1),
    };
    for (const sconv_desc_t& e : edge) {
        for (int pooled = 0; pooled < 2; ++pooled) {
            int rc = sconv_output_dims(&e, &oh, &ow, &ph, &pw);
            EXPECT(rc == SCONV_OK || rc == SCONV_EINVAL || rc == SCONV_EUNSUPPORTED);
            rc = sconv_encode_sizes(&e, pooled, &rows, &slots);
            EXPECT(rc == SCONV_OK || rc == SCONV_EINVAL || rc == SCONV_EUNSUPPORTED);
            rc = sconv_workspace_size(&e, pooled, &bytes);
            EXPECT(rc == SCONV_OK || rc == SCONV_EINVAL || rc == SCONV_EUNSUPPORTED);
            rc = sconv_filter_prep_size(&e, &bytes);
            EXPECT(rc == SCONV_OK || rc == SCONV_EINVAL || rc == SCONV_EUNSUPPORTED);
            (void)sconv_variant_name(&e, pooled);
            (void)sconv_plan_name(&e, pooled, name, sizeof(name));
        }
    }

    // invalid descriptors reach no launcher
    sconv_desc_t bad[] = {
        desc(0, 16, 8, 8, 32, 3, 3, 1, 1, 1), desc(1, 0, 8, 8, 32, 3, 3, 1, 1, 1), desc(1, 16, -1, 8, 32, 3, 3, 1, 1, 1),
        desc(1, 16, 8, 8, 0, 3, 3, 1, 1, 1),  desc(1, 16, 8, 8, 32, 0, 3, 1, 1, 1), desc(1, 16, 8, 8, 32, 3, 3, 0, 1, 1),
        desc(1, 16, 8, 8, 32, 3, 3, 1, -1, 1), desc(1, 16, 8, 8, 32, 3, 3, 1, 1, 0), desc(1, 16, 8, 8, 32, 3, 3, 1, 1, 3),
        desc(1, 16, 8, 8, 30, 3, 3, 1, 1, 4), desc(1, 16, 8, 8, 32, 3, 3, 1, 3, 1), desc(1, 16, 8, 8, 32, 3, 3, 1, 1, 1, 0, 0, 0, 4),
        desc(1, 16, 1, 8, 32, 3, 3, 1, 0, 1),
    };
    for (const sconv_desc_t& b : bad) {
        EXPECT(sconv_output_dims(&b, &oh, &ow, nullptr, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_forward(&b, ffake, ffake, ffake, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_forward_ws(&b, ffake, ffake, ffake, nullptr, 0, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_forward_bias(&b, ffake, ffake, ffake, ffake, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_forward_static(&b, ffake, ffake, ffake, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_forward_prep(&b, ffake, ffake, nullptr, 0, nullptr, ffake, nullptr, 0, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_encode(&b, SCONV_FMT_ECR, ffake, ffake, (int32_t*)fake, (int32_t*)fake, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_tune(&b, 0, ffake, ffake, ffake, nullptr, 0, nullptr, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_density(&b, ffake, (unsigned long long*)fake, nullptr) == SCONV_EINVAL);
        EXPECT(sconv_variant_name(&b, 0) == nullptr);
        EXPECT(sconv_plan_name(&b, 0, name, sizeof(name)) == SCONV_EINVAL);
        EXPECT(sconv_workspace_size(&b, 0, &bytes) == SCONV_EINVAL);
        EXPECT(sconv_filter_prep_size(&b, &bytes) == SCONV_EINVAL);
    }

    // null and malformed operands of valid descriptors
    sconv_desc_t g = desc(1, 128, 14, 14, 192, 3, 3, 1, 1, 2, 2, 2, 2);
    EXPECT(sconv_forward(&g, nullptr, ffake, ffake, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_pool_forward(&g, ffake, nullptr, ffake, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_pool_forward_bias(&g, ffake, ffake, nullptr, ffake, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_forward_ws(&g, ffake, ffake, ffake, fake, 0, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_pool_forward_ws(&g, ffake, ffake, ffake, reinterpret_cast<void*>(uintptr_t(260)), 1024, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_maxpool(&g, nullptr, ffake, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_set_workspace(fake, 0, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_tune(&g, 1, ffake, ffake, ffake, fake, 0, nullptr, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_filter_prep_size(&g, &bytes) == SCONV_OK && bytes == size_t(2) * 2 * (64 * 9) * 64 * 4);
    EXPECT(sconv_filter_prep(&g, ffake, fake, bytes - 1, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_pool_forward_prep(&g, ffake, ffake, fake, bytes - 256, nullptr, ffake, nullptr, 0, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_tune_prep(&g, 1, ffake, ffake, fake, 0, ffake, nullptr, 0, nullptr, 0, nullptr, nullptr) == SCONV_EINVAL);
    sconv_desc_t l1 = desc(1, 1, 28, 28, 20, 5, 5, 1, 0, 1, 2, 2, 2), l2 = desc(1, 21, 12, 12, 50, 5, 5, 1, 0, 1, 2, 2, 2);
    EXPECT(sconv_pair_forward(&l1, &l2, ffake, ffake, nullptr, ffake, nullptr, nullptr, ffake, nullptr) == SCONV_EINVAL);
    EXPECT(sconv_pair_forward(&l1, nullptr, ffake, ffake, nullptr, ffake, nullptr, nullptr, ffake, nullptr) == SCONV_EINVAL);

    // naming and sizes over a spread of ordinary shapes (planning code, cost models, string formatting)
    const int shapes[][10] = {
        {8, 256, 56, 56, 256, 3, 3, 1, 1, 1}, {8, 512, 28, 28, 512, 3, 3, 1, 1, 1}, {1, 512, 7, 7, 512, 3, 3, 1, 1, 1},
        {32, 256, 56, 56, 64, 1, 1, 1, 0, 1}, {32, 128, 56, 56, 128, 3, 3, 2, 1, 1}, {32, 896, 14, 14, 896, 3, 3, 1, 1, 7},
        {32, 48, 7, 7, 128, 5, 5, 1, 2, 1}, {1, 3, 224, 224, 64, 7, 7, 2, 3, 1}, {4, 20, 11, 11, 50, 5, 5, 1, 0, 1},
        {2, 24, 9, 13, 40, 3, 5, 3, 1, 2}, {1, 64, 17, 17, 64, 17, 17, 1, 8, 1},
    };
    for (const auto& s : shapes) {
        for (int pooled = 0; pooled < 2; ++pooled) {
            for (int flags : {0, (int)SCONV_RELU, (int)(SCONV_RELU | SCONV_ZERO_RATIO(0.3)), (int)SCONV_ZERO_RATIO(0.95),
                              (int)(SCONV_PREPARED_FILTERS | SCONV_ZERO_RATIO(0.8))}) {
                sconv_desc_t q = desc(s[0], s[1], s[2], s[3], s[4], s[5], s[6], s[7], s[8], s[9], pooled ? 2 : 0,
                                      pooled ? 2 : 0, pooled ? 2 : 0, flags);
                if (sconv_output_dims(&q, &oh, &ow, &ph, &pw) != SCONV_OK) continue;
                const char* v = sconv_variant_name(&q, pooled);
                EXPECT(v != nullptr && strlen(v) > 2);
                EXPECT(sconv_plan_name(&q, pooled, name, sizeof(name)) == SCONV_OK && strlen(name) > 2);
                EXPECT(sconv_plan_name(&q, pooled, name, 4) == SCONV_OK && strlen(name) <= 3);   // truncated, terminated
                EXPECT(sconv_workspace_size(&q, pooled, &bytes) == SCONV_OK);
                EXPECT(sconv_filter_prep_size(&q, &bytes) == SCONV_OK);
            }
        }
    }
    EXPECT(sconv_plan_name(&g, 1, nullptr, 10) == SCONV_EINVAL && sconv_plan_name(&g, 1, name, 0) == SCONV_EINVAL);

    // the plan table as text
    {
        EXPECT(sconv_tune_reset() == SCONV_OK);
        const char* line = "sconv-plan 1 8 256 56 56 256 3 3 1 1 1 0 0 0 1 0 0 0 2 1 q32t7d 8 4 0 0.24 quad3x3/q32t7d/8x4\n";
        EXPECT(sconv_tune_import(line) == SCONV_OK);
        size_t need = 0;
        EXPECT(sconv_tune_export(nullptr, 0, &need) == SCONV_OK && need == strlen(line) + 1);
        char buf[256];
        EXPECT(sconv_tune_export(buf, sizeof(buf), nullptr) == SCONV_OK && strcmp(buf, line) == 0);
        EXPECT(sconv_tune_export(buf, 5, nullptr) == SCONV_EINVAL);
        sconv_desc_t q = desc(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 0, 0, 0, SCONV_RELU);
        EXPECT(sconv_plan_name(&q, 0, name, sizeof(name)) == SCONV_OK && strcmp(name, "quad3x3/q32t7d/8x4") == 0);
        const char* junk[] = {"", "\n\n", "sconv-plan", "sconv-plan 1", "sconv-plan 1 1 2 3", "sconv-plan 7 x",
                              "sconv-plan 1 8 256 56 56 256 3 3 1 1 1 0 0 0 1 0 0 0 2 1 nosuchgeometrynamethatistoolongtofit 8 4 0 0.2 n",
                              "sconv-plan 1 8 256 56 56 256 3 3 1 1 1 0 0 0 1 0 0 0 -3 1 - 8 4 0 0.2 n",
                              "sconv-plan 1 8 256 56 56 256 3 3 1 1 1 0 0 0 1 0 0 0 2 1 - 2147483647 4 0 0.2 n"};
        for (const char* j : junk) {
            const int rc = sconv_tune_import(j);
            EXPECT(rc == SCONV_OK || rc == SCONV_EINVAL);
        }
        EXPECT(sconv_tune_import(nullptr) == SCONV_EINVAL);
        EXPECT(sconv_tune_reset() == SCONV_OK);
    }

    // process-state calls that need no device
    EXPECT(sconv_env_refresh() == SCONV_OK);
    EXPECT(sconv_tune_reset() == SCONV_OK);
    EXPECT(sconv_clear_workspaces() == SCONV_OK);
    for (int code = 1; code >= -6; --code) EXPECT(sconv_strerror(code) != nullptr && strlen(sconv_strerror(code)) > 3);

    if (failures) {
        fprintf(stderr, "%d expectation(s) failed\n", failures);
        return 1;
    }
    printf("ok\n");
    return 0;
}
