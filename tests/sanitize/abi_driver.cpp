// Calls the C ABI's host-side logic -- the shape planning behind the workspace and path queries, and the argument
// validation of every entry point (calls that must fail before any HIP call) -- in a build whose host code runs
// under -fsanitize=address,undefined (tests/test_sanitizers.py).  No GPU is touched.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "dropit.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); std::exit(3); } } while (0)

int main()
{
    CHECK(dropit_keep_count(16384, 0.9) == 1638);
    CHECK(dropit_keep_count(-1, 0.5) == -1 && dropit_keep_count(10, std::nan("")) == -1);
    for (int s = 0; s < 5; ++s) CHECK(dropit_status_string(static_cast<dropit_status>(s)) != nullptr);
    CHECK(dropit_status_string(static_cast<dropit_status>(99)) != nullptr);

    // ---- planning: every path, small and extreme shapes ----
    const int64_t fc_shapes[][3] = {{1, 8, 8}, {256, 64, 128}, {12608, 768, 3072}, {12608, 3072, 768}, {16384, 3072, 768},
                                    {777, 257, 33}, {640, 40000, 8}, {70000, 64, 8}, {2147483647LL / 8, 8, 8}, {5, 24, 16},
                                    {1, 1, 1}, {33, 496, 3}, {2000, 3000, 8}};
    size_t total = 0;
    for (const auto &s : fc_shapes) {
        const int64_t shape[2] = {s[0], s[1]};
        for (int dt = 0; dt < 2; ++dt) {
            const int64_t k = dropit_keep_count(s[0] * s[1], 0.9);
            total += dropit_weight_grad_workspace_bytes(shape, 2, static_cast<dropit_dtype>(dt), k, s[2], nullptr);
            total += dropit_weight_grad_path(shape, 2, static_cast<dropit_dtype>(dt), k, s[2], nullptr);
            total += dropit_weight_grad_rows_workspace_bytes(shape, 2, static_cast<dropit_dtype>(dt), k, s[2], nullptr);
            total += dropit_weight_grad_mask_workspace_bytes(shape, 2, static_cast<dropit_dtype>(dt), k, s[2], nullptr);
            total += dropit_compress_workspace_bytes(s[0] * s[1], static_cast<dropit_dtype>(dt));
            total += dropit_compress_random_workspace_bytes(s[0] * s[1], static_cast<dropit_dtype>(dt));
            total += dropit_compress_rows_workspace_bytes(s[0] * s[1], k, static_cast<dropit_dtype>(dt));
            total += dropit_compress_mask_workspace_bytes(s[0] * s[1], k, static_cast<dropit_dtype>(dt));
        }
    }
    const int64_t conv_shapes[][5] = {{64, 64, 56, 56, 64}, {2, 5, 9, 11, 7}, {1, 1, 3, 3, 1}, {64, 128, 28, 28, 128},
                                      {64, 256, 14, 14, 256}, {64, 512, 7, 7, 512}, {600, 64, 7, 7, 64}, {1, 3, 61, 120, 5},
                                      {3, 16, 9, 1, 8}, {64, 3, 224, 224, 64}, {2, 4096, 7, 7, 64}, {1, 8, 1, 1, 8}};
    const dropit_conv2d geoms[] = {{3, 3, 1, 1, 1, 1, 1, 1}, {1, 1, 1, 1, 0, 0, 1, 1}, {7, 7, 2, 2, 3, 3, 1, 1}, {3, 3, 2, 2, 1, 1, 1, 1},
                                   {16, 16, 16, 16, 0, 0, 1, 1}, {3, 2, 1, 2, 2, 0, 2, 3}, {3, 3, 1, 1, 4, 4, 1, 1},
                                   {1024, 1024, 65535, 65535, 65535, 65535, 65535, 65535}, {1025, 1, 1, 1, 0, 0, 1, 1}, {0, 3, 1, 1, 1, 1, 1, 1}};
    for (const auto &s : conv_shapes)
        for (const auto &g : geoms)
            for (int dt = 0; dt < 2; ++dt) {
                const int64_t nchw[4] = {s[0], s[1], s[2], s[3]}, nhwc[4] = {s[0], s[2], s[3], s[1]};
                const int64_t k = dropit_keep_count(s[0] * s[1] * s[2] * s[3], 0.8);
                total += dropit_weight_grad_workspace_bytes(nchw, 4, static_cast<dropit_dtype>(dt), k, s[4], &g);
                total += dropit_weight_grad_path(nchw, 4, static_cast<dropit_dtype>(dt), k, s[4], &g);
                total += dropit_weight_grad_nhwc_workspace_bytes(nhwc, static_cast<dropit_dtype>(dt), k, s[4], &g);
                total += dropit_weight_grad_nhwc_path(nhwc, static_cast<dropit_dtype>(dt), k, s[4], &g);
                total += dropit_weight_grad_rows_workspace_bytes(nchw, 4, static_cast<dropit_dtype>(dt), k, s[4], &g);
                total += dropit_weight_grad_mask_workspace_bytes(nchw, 4, static_cast<dropit_dtype>(dt), k, s[4], &g);
            }

    // ---- validation: each of these must be refused before any HIP call ----
    void *fake = reinterpret_cast<void *>(0x1000), *ws = reinterpret_cast<void *>(0x10000);
    int32_t *ifake = reinterpret_cast<int32_t *>(0x2000);
    float *ffake = reinterpret_cast<float *>(0x3000);
    const int64_t s44[2] = {4, 4}, bad0[2] = {4, 0}, huge[2] = {int64_t(1) << 20, int64_t(1) << 12};
    const size_t big = size_t(1) << 40;
    CHECK(dropit_compress(nullptr, s44, 2, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, nullptr, 2, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 0, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, bad0, 2, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, huge, 2, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 2, static_cast<dropit_dtype>(7), 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 2, DROPIT_BF16, std::nan(""), fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(reinterpret_cast<void *>(0x1004), s44, 2, DROPIT_BF16, 0.5, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 2, DROPIT_BF16, 0.5, nullptr, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 2, DROPIT_BF16, 0.5, fake, ifake, reinterpret_cast<void *>(0x10010), big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress(fake, s44, 2, DROPIT_BF16, 0.5, fake, ifake, ws, 16, nullptr) == DROPIT_EWORKSPACE);
    CHECK(dropit_compress(fake, s44, 2, DROPIT_BF16, 1.0, nullptr, nullptr, nullptr, 0, nullptr) == DROPIT_OK);   // k = 0: nothing to do
    CHECK(dropit_compress_static(nullptr, s44, 2, DROPIT_BF16, 0.5, fake, ifake, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress_static(fake, huge, 2, DROPIT_BF16, 0.5, fake, ifake, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress_random(fake, s44, 2, DROPIT_BF16, 2.0, 1, fake, ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress_random(fake, s44, 2, DROPIT_BF16, 0.5, 1, fake, ifake, ws, 16, nullptr) == DROPIT_EWORKSPACE);
    CHECK(dropit_compress_rows(nullptr, s44, 2, DROPIT_BF16, 0.5, fake, reinterpret_cast<uint16_t *>(fake), ifake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_compress_mask(nullptr, s44, 2, DROPIT_BF16, 0.5, fake, reinterpret_cast<uint32_t *>(fake), ifake, ws, big, nullptr) == DROPIT_EINVAL);
    const dropit_conv2d c3 = {3, 3, 1, 1, 1, 1, 1, 1}, window = {7, 7, 1, 1, 0, 0, 1, 1};
    const int64_t x4[4] = {1, 2, 4, 4};
    CHECK(dropit_weight_grad(fake, ifake, 99, s44, 2, DROPIT_BF16, fake, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);   // k > numel
    CHECK(dropit_weight_grad(nullptr, ifake, 4, s44, 2, DROPIT_BF16, fake, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_weight_grad(fake, ifake, 4, s44, 2, DROPIT_BF16, nullptr, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_weight_grad(fake, ifake, 4, s44, 2, DROPIT_BF16, fake, 0, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_weight_grad(fake, ifake, 4, s44, 2, DROPIT_BF16, fake, 8, &c3, ffake, ws, big, nullptr) == DROPIT_EINVAL);      // conv needs 4 dims
    CHECK(dropit_weight_grad(fake, ifake, 4, x4, 4, DROPIT_BF16, fake, 8, &window, ffake, ws, big, nullptr) == DROPIT_EINVAL);   // window larger than the input
    CHECK(dropit_weight_grad(fake, ifake, 4, x4, 4, DROPIT_BF16, fake, 8, &c3, ffake, ws, 0, nullptr) == DROPIT_EWORKSPACE);
    CHECK(dropit_weight_grad_nhwc(fake, ifake, 4, x4, DROPIT_BF16, fake, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_weight_grad_rows(fake, nullptr, ifake, 4, s44, 2, DROPIT_BF16, fake, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_weight_grad_mask(fake, nullptr, ifake, 4, s44, 2, DROPIT_BF16, fake, 8, nullptr, ffake, ws, big, nullptr) == DROPIT_EINVAL);
    CHECK(dropit_set_select_mode(9) == DROPIT_EINVAL && dropit_set_select_mode(0) == DROPIT_OK);
    dropit_trace_events(nullptr, 0);
    std::printf("ABI host logic under sanitizers: OK (%zu)\n", total);
    return 0;
}
