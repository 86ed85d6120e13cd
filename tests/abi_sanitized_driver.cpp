// Host side of libef under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): built by
// tests/test_abi_sanitized.py from csrc/ef_api.hip plus this file.  It walks the argument checks of every
// entry point, which return before any GPU work, and the creation / destruction of a plan: without a GPU
// creation fails after the host-side set-up and must release everything it took; with one, the host-side
// lists behind ef_plan_tune, ef_plan_set_persistent and ef_plan_set_lazy are rebuilt a few times.
// Test infrastructure only.
#include "ef.h"
#include "ef_debug.h"

#include <cstdio>
#include <cstring>
#include <vector>

#define REQUIRE(cond)                                                  \
    do {                                                               \
        if (!(cond)) {                                                 \
            std::fprintf(stderr, "line %d: %s failed\n", __LINE__, #cond); \
            return 1;                                                  \
        }                                                              \
    } while (0)

int main()
{
    ef_plan *p = nullptr;
    float ms = 0.f;
    unsigned int a = 0, b = 0;
    double q[2];
    alignas(16) static float buf[64];
    alignas(16) static uint64_t words[8];

    // partitions that must be refused before any GPU call
    const int64_t empty_block[3] = {0, 2, 2}, not_from_zero[3] = {1, 2, 3}, decreasing[3] = {0, 3, 2};
    REQUIRE(ef_plan_create(&p, empty_block, 2, 4, nullptr) == EF_ERR_OFFSETS && p == nullptr);
    REQUIRE(ef_plan_create(&p, not_from_zero, 2, 4, nullptr) == EF_ERR_OFFSETS);
    REQUIRE(ef_plan_create(&p, decreasing, 2, 4, nullptr) == EF_ERR_OFFSETS);
    REQUIRE(ef_plan_create(&p, nullptr, 2, 4, nullptr) != EF_OK);
    REQUIRE(ef_plan_create(nullptr, empty_block, 2, 4, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_plan_create(&p, empty_block, 0, 4, nullptr) != EF_OK);
    const int64_t good[4] = {0, 5000, 9000, 9001};
    REQUIRE(ef_plan_create(&p, good, 3, 0, nullptr) == EF_ERR_ARG);
    REQUIRE(ef_plan_create(&p, good, 3, EF_MAX_WORKERS + 1, nullptr) == EF_ERR_ARG);

    // a missing plan is an error everywhere, never a crash
    REQUIRE(ef_plan_destroy(nullptr) == EF_ERR_NULL);
    REQUIRE(ef_plan_tune(nullptr, 1, 1) == EF_ERR_NULL);
    REQUIRE(ef_plan_set_persistent(nullptr, 1) == EF_ERR_NULL);
    REQUIRE(ef_plan_set_lazy(nullptr, 1) == EF_ERR_NULL);
    REQUIRE(ef_plan_set_sync_group(nullptr, 16) == EF_ERR_NULL);
    REQUIRE(ef_plan_last_fallbacks(nullptr, &a, &b) == EF_ERR_NULL);
    REQUIRE(ef_plan_fuse_limit(nullptr) == 0 && ef_plan_is_persistent(nullptr) == 0 && ef_plan_is_lazy(nullptr) == 0);
    REQUIRE(ef_plan_d(nullptr) == 0 && ef_plan_blocks(nullptr) == 0 && ef_sign_words(nullptr) == 0);
    REQUIRE(ef_payload_bytes(nullptr) == 0 && ef_payload_scales_offset(nullptr) == 0);
    REQUIRE(ef_worker_step(nullptr, 1, buf, 64, buf, buf, 64, 0.9f, 0.f, 0.1f, words, buf, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_worker_step_quality(nullptr, 1, buf, 64, buf, buf, 64, 0.9f, 0.f, 0.1f, words, buf, q, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_worker_step_sgd(nullptr, 1, buf, 64, buf, 64, 0.f, 0.1f, words, buf, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_server_step(nullptr, 1, words, buf, buf, 0.f, 0.1f, words, buf, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_apply(nullptr, buf, words, buf, 0.1f, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_apply_wd(nullptr, buf, buf, words, buf, 0.1f, 0.9f, 0.f, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_worker_step_fused(nullptr, 1, buf, 64, buf, buf, 64, 0.9f, 0.f, 0.1f, words, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_server_step_fused(nullptr, 1, words, buf, 0.f, 0.1f, words, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_apply_fused(nullptr, buf, words, 0.1f, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_flush(nullptr, 1, buf, 64, buf, nullptr) == EF_ERR_NULL);
    {
        ef_state *st = nullptr;
        REQUIRE(ef_state_create(nullptr, 1, &st, nullptr) == EF_ERR_NULL && st == nullptr);
        REQUIRE(ef_state_destroy(nullptr) == EF_ERR_NULL);
        REQUIRE(ef_worker_step_state(nullptr, nullptr, buf, 64, 0.9f, 0.f, 0.1f, words, buf, nullptr) == EF_ERR_NULL);
        REQUIRE(ef_server_step_state(nullptr, nullptr, 1, words, buf, 0.f, 0.1f, words, buf, nullptr) == EF_ERR_NULL);
        REQUIRE(ef_state_export(nullptr, nullptr, buf, buf, 64, buf, nullptr) == EF_ERR_NULL);
        REQUIRE(ef_state_import(nullptr, nullptr, buf, buf, 64, buf, nullptr) == EF_ERR_NULL);
    }
    REQUIRE(ef_compressor_quality(nullptr, 1, buf, 64, q, nullptr) == EF_ERR_NULL);
    REQUIRE(ef_compressor_quality_static(nullptr, 1, buf, 64, q, nullptr) == EF_ERR_NULL);

    for (int code = 1; code >= -7; --code) REQUIRE(ef_strerror(code) != nullptr && std::strlen(ef_strerror(code)) > 0);

    // a real layout: many tiny blocks, blocks of several tiles, a ragged end
    std::vector<int64_t> offs(1, 0);
    for (int k = 0; k < 3000; ++k) offs.push_back(offs.back() + 1 + k % 7);
    for (int k = 0; k < 5; ++k) offs.push_back(offs.back() + 4096 * (k + 1) + k);
    offs.push_back(offs.back() + 100000);
    const int rc = ef_plan_create(&p, offs.data(), (int64_t)offs.size() - 1, 3, nullptr);
    if (rc == EF_ERR_HIP) {
        REQUIRE(p == nullptr);
        std::printf("no GPU: plan creation refused after host set-up (%s)\n", ef_strerror(rc));
    } else {
        REQUIRE(rc == EF_OK && p != nullptr);
        REQUIRE(ef_plan_d(p) == offs.back() && ef_plan_blocks(p) == (int64_t)offs.size() - 1);
        for (int lim = 0; lim < 6; ++lim) {
            REQUIRE(ef_plan_tune(p, lim, -1) == EF_OK && ef_plan_fuse_limit(p) == lim);
            REQUIRE(ef_plan_set_persistent(p, lim & 1) == EF_OK);
            REQUIRE(ef_plan_set_lazy(p, (lim >> 1) & 1) == EF_OK);
            REQUIRE(ef_plan_set_sync_group(p, lim * 3) == EF_OK);
        }
        REQUIRE(ef_plan_set_persistent(p, -1) == EF_OK);
        REQUIRE(ef_flush(p, 1, nullptr, 0, nullptr, nullptr) == EF_OK);
        REQUIRE(ef_plan_last_fallbacks(p, &a, &b) == EF_OK);
        REQUIRE(ef_plan_destroy(p) == EF_OK);
        std::printf("GPU present: plan created, lists rebuilt, destroyed\n");
    }
    std::puts("abi sanitized run ok");
    return 0;
}
