// Host side of the C ABI under AddressSanitizer / UBSan (no GPU needed): every entry point is called
// with arguments that the validation layer must refuse before anything is launched, the host-only
// helpers are exercised, and a few valid calls run the launch planning up to the first launch (which
// a machine without a GPU refuses: DLION_ELAUNCH).  Built and run by tests/test_sanitizers.py.
#include "../include/dlion.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static int failures = 0;
#define EXPECT(expr, want)                                                                      \
    do {                                                                                        \
        const long got_ = (long)(expr);                                                         \
        if (got_ != (long)(want)) {                                                             \
            std::fprintf(stderr, "%s:%d: %s = %ld, expected %ld\n", __FILE__, __LINE__, #expr, got_, (long)(want)); \
            ++failures;                                                                         \
        }                                                                                       \
    } while (0)

int main()
{
    // a 256-byte aligned fake device address; validation never dereferences device pointers
    char *const A = reinterpret_cast<char *>(0x7F0000000000ull);
    float *const fA = reinterpret_cast<float *>(A);
    uint64_t *const pA = reinterpret_cast<uint64_t *>(A);
    uint16_t *const cA = reinterpret_cast<uint16_t *>(A);

    EXPECT(dlion_worker_step(fA, 128, A, 128, DLION_F32, pA, 2, 0, 4, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step(fA, 128, A, 128, DLION_F32, pA, 2, 128, 65536, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step(nullptr, 128, A, 128, DLION_F32, pA, 2, 128, 4, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step(fA, 127, A, 128, DLION_F32, pA, 2, 128, 4, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step(fA, 128, A, 128, (dlion_dtype)7, pA, 2, 128, 4, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step(reinterpret_cast<float *>(A + 2), 128, A, 128, DLION_F32, pA, 2, 128, 4, 0.9f, 0.99f, nullptr), DLION_EALIGN);
    EXPECT(dlion_worker_step(fA, 128, A + 1, 128, DLION_BF16, pA, 2, 128, 4, 0.9f, 0.99f, nullptr), DLION_EALIGN);
    EXPECT(dlion_aggregate(pA, 2, 128, 4, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_aggregate(pA, 1, 128, 4, cA, nullptr), DLION_EINVAL);
    EXPECT(dlion_aggregate(pA, 2, 128, 4, reinterpret_cast<uint16_t *>(A + 1), nullptr), DLION_EALIGN);
    EXPECT(dlion_apply(nullptr, cA, 128, 4, DLION_VOTE, 1e-4f, 0.1f, nullptr), DLION_EINVAL);
    EXPECT(dlion_apply(fA, cA, 128, 4, (dlion_mode)2, 1e-4f, 0.1f, nullptr), DLION_EINVAL);
    EXPECT(dlion_aggregate_apply(fA, pA, 1, 128, 4, DLION_VOTE, 1e-4f, 0.1f, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_step(nullptr, fA, 128, A, 128, DLION_F32, 128, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_step(fA, fA, 64, A, 128, DLION_F32, 128, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_step_ws(fA, fA, 1024, A, 1024, DLION_F32, 1024, 4, DLION_VOTE, 0.9f, 0.99f, 1e-3f, 0.1f, nullptr, 0, nullptr, A, -1, nullptr), DLION_EINVAL);
    EXPECT(dlion_step_ws(fA, fA, 1024, A, 1024, DLION_F32, 1024, 4, DLION_VOTE, 0.9f, 0.99f, 1e-3f, 0.1f, nullptr, 0, nullptr, nullptr, 64, nullptr), DLION_EINVAL);
    EXPECT(dlion_step_ws(fA, fA, 1024, A, 1024, DLION_F32, 1024, 4, DLION_VOTE, 0.9f, 0.99f, 1e-3f, 0.1f, nullptr, 0, nullptr, A + 8, 4096, nullptr), DLION_EALIGN);
    EXPECT(dlion_step_noalloc(nullptr, fA, 128, A, 128, DLION_F32, 128, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_step_noalloc(fA, fA, 128, A, 128, DLION_F32, 0, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_aggregate_encode(pA, 2, 128, 4, DLION_VOTE, pA, 1, nullptr), DLION_EINVAL);
    EXPECT(dlion_apply_encoded(fA, pA, 1, 128, 4, DLION_AVG, 1e-4f, 0.1f, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step_pw(fA, 128, A, 128, DLION_F32, pA, 2, 128, 4, nullptr, fA, nullptr), DLION_EINVAL);
    EXPECT(dlion_step_pw(fA, fA, 128, A, 128, DLION_F32, 128, 4, DLION_VOTE, nullptr, fA, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_global_lion_step(fA, fA, 100, A, 128, DLION_F32, 128, 4, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, nullptr), DLION_EINVAL);
        EXPECT(dlion_membench(A, 4096, 2, A, 1000, 1, 16, 0, nullptr), DLION_EINVAL);
    EXPECT(dlion_membench(A + 4, 4096, 1, A, 1024, 1, 16, 0, nullptr), DLION_EALIGN);

    // host-only helpers
    EXPECT(dlion_delta_planes(3, DLION_VOTE), 1);
    EXPECT(dlion_delta_planes(4, DLION_VOTE), 2);
    EXPECT(dlion_delta_planes(65535, DLION_AVG), 16);
    EXPECT(dlion_delta_planes(0, DLION_AVG), 0);
    EXPECT(dlion_step_workspace_bytes(350000000, 32), 262144L * 3 * 128);
    EXPECT(dlion_step_workspace_bytes(-5, 32), 0);
    EXPECT(dlion_step_mt_workspace_bytes(1L << 31, 32), 0);
    EXPECT(std::strlen(dlion_status_str(DLION_EALIGN)) > 0, 1);
    EXPECT(std::strcmp(dlion_status_str((dlion_status)99), "unknown status"), 0);

    // tensor-list layout and validation (host table on the heap so that overruns would be seen)
    const int64_t numels[] = {64, 1000, 5, 256, 257};
    std::vector<dlion_seg> segs(5);
    for (int k = 0; k < 5; ++k) {
        segs[k].x = fA;
        segs[k].m = fA;
        segs[k].g = A;
        segs[k].m_stride = segs[k].g_stride = numels[k];
        segs[k].numel = numels[k];
        segs[k].word_begin = segs[k].tile_begin = -1;
    }
    int64_t words = 0, tiles = 0;
    EXPECT(dlion_mt_layout(segs.data(), 5, &words, &tiles), DLION_OK);
    EXPECT(words, 1 + 16 + 1 + 4 + 5);
    EXPECT(tiles, 1 + 4 + 1 + 1 + 2);
    EXPECT(segs[4].word_begin, 22);
    EXPECT(segs[4].tile_begin, 7);
    const dlion_seg *dev = reinterpret_cast<const dlion_seg *>(A);
    segs[3].word_begin += 1;
    EXPECT(dlion_step_mt(segs.data(), dev, 5, DLION_F32, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_EINVAL);
    segs[3].word_begin -= 1;
    EXPECT(dlion_step_mt_ws(segs.data(), dev, 5, DLION_F32, 4, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, A + 8, 4096, nullptr), DLION_EALIGN);
    EXPECT(dlion_aggregate_mt(segs.data(), dev, 5, pA, 2, 4, cA, nullptr), DLION_EINVAL);     // packed stride < total words
    EXPECT(dlion_apply_mt(segs.data(), dev, 5, nullptr, 4, DLION_VOTE, 1e-4f, 0.1f, nullptr), DLION_EINVAL);
    EXPECT(dlion_aggregate_apply_mt(segs.data(), dev, 5, pA, 64, 4, (dlion_mode)3, 1e-4f, 0.1f, nullptr, nullptr), DLION_EINVAL);
    EXPECT(dlion_worker_step_mt(segs.data(), nullptr, 5, DLION_F32, pA, 64, 4, 0.9f, 0.99f, nullptr), DLION_EINVAL);
    segs[2].numel = 0;
    EXPECT(dlion_mt_layout(segs.data(), 5, nullptr, nullptr), DLION_EINVAL);
    segs[2].numel = 5;

    // tuning: validation, and the launch planning of valid calls with and without overrides.  Without a
    // GPU the first launch is refused, after the plan (blocks, launches, hand-over format) has been made.
    dlion_tuning t;
    dlion_tuning_defaults(&t);
    EXPECT(t.unroll, -1);
    EXPECT(t.block_tiles, -1);
    t.unroll = 3;
    EXPECT(dlion_set_tuning(&t), DLION_EINVAL);
    t.unroll = 2;
    t.pass_workers = 3;
    t.block_tiles = 5;
    EXPECT(dlion_set_tuning(&t), DLION_OK);
    dlion_tuning back;
    dlion_get_tuning(&back);
    EXPECT(back.pass_workers, 3);
    EXPECT(dlion_step_workspace_bytes(70001, 33), 5 * 512);
    const bool has_gpu = std::getenv("DLION_SANITIZE_EXPECT_GPU") != nullptr;
    if (!has_gpu) {
        for (int32_t N : {1, 4, 9, 33, 70}) {
            EXPECT(dlion_step_ws(fA, fA, 70016, A, 70016, DLION_BF16, 70001, N, DLION_AVG, 0.9f, 0.99f, 1e-4f, 0.1f, pA, 1100, cA, A, 1 << 20, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_step(fA, fA, 70016, A, 70016, DLION_F32, 70001, N, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_worker_step(fA, 70016, A, 70016, DLION_F32, pA, 1100, 70001, N, 0.9f, 0.99f, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_aggregate(pA, 1100, 70001, N, cA, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_aggregate_apply(fA, pA, 1100, 70001, N, DLION_AVG, 1e-4f, 0.1f, cA, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_aggregate_encode(pA, 1100, 70001, N, DLION_AVG, pA, 1100, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_apply_encoded(fA, pA, 1100, 70001, N, DLION_VOTE, 1e-4f, 0.1f, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_membench(A, 4096, N, A, 4096, 1, 4, 0, nullptr), DLION_ELAUNCH);
            EXPECT(dlion_membench(A, 4096, N, A, 4096, 1, 3, 0, nullptr), DLION_EINVAL);
        }
        EXPECT(dlion_step_mt_ws(segs.data(), dev, 5, DLION_F32, 20, DLION_VOTE, 0.9f, 0.99f, 1e-4f, 0.1f, nullptr, 0, nullptr, A, 1 << 20, nullptr), DLION_ELAUNCH);
    }
    EXPECT(dlion_set_tuning(nullptr), DLION_OK);
    dlion_get_tuning(&back);
    EXPECT(back.pass_workers, -1);

    if (failures)
        std::fprintf(stderr, "%d expectation(s) failed\n", failures);
    else
        std::printf("host layer ok\n");
    return failures ? 1 : 0;
}
