// Host-side check of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer: every entry point's argument
// validation, workspace arithmetic and error text, on a machine with or without a GPU.  Built by
// `python -m paper_2210_17323_amd.build --host-sanitize` (host code instrumented, device code as usual) and run by
// tests/test_host_sanitizers.py.  No call here reaches a kernel launch with usable pointers: calls that pass validation
// are only made with sizes of zero, or expect GPTQ_ERR_HIP / GPTQ_ERR_WORKSPACE before anything is enqueued.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>

#include "../include/gptq.h"

static int g_failed = 0;
#define EXPECT(cond)                                                                  \
    do {                                                                              \
        if (!(cond)) { std::printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, gptq_last_error()); ++g_failed; } \
    } while (0)

int main() {
    alignas(256) static unsigned char buf[4096];
    void* one = buf;
    void* odd = buf + 4;
    const size_t big = (size_t)1 << 40;

    EXPECT(gptq_version() >= 100);
    EXPECT(gptq_release_thread_resources() == GPTQ_OK);
    // sizes over the whole range of shapes, including the largest workload and degenerate ones
    for (int64_t n : {(int64_t)0, (int64_t)1, (int64_t)127, (int64_t)4096, (int64_t)14336, (int64_t)49152, (int64_t)1 << 20}) {
        (void)gptq_damp_cholesky_inverse_workspace_bytes(n);
        (void)gptq_damp_cholesky_workspace_bytes(n);
        (void)gptq_symmetric_update_split_workspace_bytes(n);
        for (int64_t r : {(int64_t)0, (int64_t)3, (int64_t)12288, (int64_t)49152}) {
            for (int64_t group : {(int64_t)0, (int64_t)8, (int64_t)128, (int64_t)1024}) (void)gptq_quantize_layer_workspace_bytes(r, n, 128, group);
            (void)gptq_trailing_update_split_workspace_bytes(r, n);
        }
        for (int64_t t : {(int64_t)0, (int64_t)1, (int64_t)160, (int64_t)32768, (int64_t)262144})
            for (int dt = 0; dt < 3; ++dt) {
                (void)gptq_hessian_accumulate_workspace_bytes(n, t, dt);
                (void)gptq_hessian_accumulate_token_major_workspace_bytes(n, t, dt);
                (void)gptq_hessian_accumulate_launches(n, t, dt);
            }
    }
    EXPECT(gptq_damp_cholesky_inverse_workspace_bytes(-5) == gptq_damp_cholesky_inverse_workspace_bytes(0));
    EXPECT(gptq_trailing_update_split_workspace_bytes(-1, 4) == 0);

    // step 1
    EXPECT(gptq_hessian_accumulate((float*)one, 8, one, 7, 8, 16, 16, nullptr, 0, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_hessian_accumulate((float*)one, 4, one, 0, 8, 16, 16, nullptr, 0, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_hessian_accumulate((float*)one, 8, one, 0, 0, 8, 8, nullptr, 0, nullptr) == GPTQ_OK);
    EXPECT(gptq_hessian_accumulate((float*)one, 49152, one, 0, 49152, 32768, 32768, one, 1024, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(gptq_hessian_accumulate((float*)one, 49152, one, 0, 49152, 32768, 32768, odd, big, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(std::strstr(gptq_last_error(), "workspace") != nullptr);
    EXPECT(gptq_hessian_accumulate_token_major((float*)one, 8, one, 2, 8, 16, 8, one, big, nullptr) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(gptq_hessian_accumulate_token_major((float*)one, 8, one, 0, 8, 16, 8, nullptr, 0, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(gptq_hessian_symmetrize(nullptr, 8, 8, nullptr) != GPTQ_OK);

    // step 2
    int* info = (int*)one;
    EXPECT(gptq_damp_cholesky_inverse((float*)one, 8, 8, -0.5f, one, big, info, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_damp_cholesky_inverse((float*)one, 8, 8, 0.01f, one, 16, info, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(gptq_damp_cholesky_inverse((float*)one, 6, 6, 0.01f, one, big, info, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_damp_cholesky((float*)one, 8, 8, 0.01f, nullptr, 0, info, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(gptq_damp_cholesky((float*)one, 8, 0, 0.01f, nullptr, 0, info, nullptr) == GPTQ_OK);
    EXPECT(gptq_damp_cholesky_inverse_noalloc((float*)one, 4100, 4100, 0.01f, info, nullptr) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(std::strstr(gptq_last_error(), "4096") != nullptr);
    EXPECT(gptq_damp_cholesky_inverse_noalloc((float*)one, 8, 8, 0.01f, nullptr, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_check_info(nullptr, nullptr, nullptr) == GPTQ_ERR_INVALID_ARG);

    // step 3
    auto q = [&](int wd, int64_t r, int bits, int grid, int block, int64_t group, void* ws, size_t wsb) {
        return gptq_quantize_layer(one, wd, 256, r, 256, (const float*)one, 256, bits, grid, block, group, (uint8_t*)one, 256, (float*)one,
                                   (int32_t*)one, nullptr, 0, nullptr, ws, wsb, nullptr);
    };
    EXPECT(q(0, 4, 5, 0, 128, 0, one, big) == GPTQ_ERR_INVALID_ARG);
    EXPECT(q(0, 4, 4, 3, 128, 0, one, big) == GPTQ_ERR_INVALID_ARG);
    EXPECT(q(0, 4, 4, 0, 64, 0, one, big) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(q(0, 4, 4, 0, 128, 100, one, big) == GPTQ_ERR_INVALID_ARG);
    EXPECT(q(0, 4, 4, 0, 128, 4, one, big) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(q(9, 4, 4, 0, 128, 0, one, big) == GPTQ_ERR_INVALID_ARG);
    EXPECT(q(0, 4, 4, 0, 128, 0, one, 1024) == GPTQ_ERR_WORKSPACE);
    EXPECT(q(0, 0, 4, 0, 128, 0, one, big) == GPTQ_OK);
    EXPECT(gptq_quantize_layer_from_factor_supports(128) == 1 && gptq_quantize_layer_from_factor_supports(8) == 0);
    EXPECT(gptq_quantize_layer_from_factor(one, 0, 256, 4, 256, (const float*)one, 256, 4, 0, 128, 8, (uint8_t*)one, 256, (float*)one, (int32_t*)one,
                                           nullptr, 0, nullptr, one, big, nullptr) == GPTQ_ERR_UNSUPPORTED);

    // deferred updates on their own
    EXPECT(gptq_trailing_update((float*)odd, 64, (const float*)one, 8, (const float*)one, 64, 4, 64, 8, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_trailing_update((float*)one, 60, (const float*)one, 8, (const float*)one, 64, 4, 64, 8, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_trailing_update((float*)one, 64, (const float*)one, 8, (const float*)one, 64, 0, 64, 8, nullptr) == GPTQ_OK);
    EXPECT(gptq_trailing_update_split((float*)one, 256, (const float*)one, 1024, (const float*)one, 256, 256, 256, 512, one, big, nullptr) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(gptq_trailing_update_split((float*)one, 256, (const float*)one, 1024, (const float*)one, 256, 256, 256, 1024, one, 1024, nullptr) == GPTQ_ERR_WORKSPACE);
    EXPECT(gptq_trailing_update_split((float*)one, 256, (const float*)one, 1024, (const float*)one, 256, 0, 256, 1024, one, big, nullptr) == GPTQ_OK);
    EXPECT(gptq_symmetric_update_split((float*)one, 256, (const float*)one, 1024, 300, 1024, one, big, nullptr) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(gptq_symmetric_update_split((float*)one, 256, (const float*)one, 1000, 256, 1024, one, big, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_symmetric_update_split((float*)one, 256, (const float*)one, 1024, 256, 1024, one, 64, nullptr) == GPTQ_ERR_WORKSPACE);
    const int prev = gptq_set_split_min_tiles(7);
    EXPECT(gptq_set_split_min_tiles(prev) == 7);

    // step 4 and the consumers
    EXPECT(gptq_pack((const uint8_t*)one, 64, 2, 64, 5, (uint32_t*)one, 8, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_pack((const uint8_t*)one, 64, 2, 64, 3, (uint32_t*)one, 5, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_pack((const uint8_t*)one, 64, 0, 64, 3, (uint32_t*)one, 6, nullptr) == GPTQ_OK);
    EXPECT(gptq_unpack((const uint32_t*)one, 6, 2, 64, 3, nullptr, 64, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_dequantize_packed((const uint32_t*)one, 5, 2, 64, 3, (const float*)one, (const int32_t*)one, 0, one, 0, 64, nullptr) == GPTQ_ERR_INVALID_ARG);
    EXPECT(gptq_dequantize_packed((const uint32_t*)one, 6, 0, 64, 3, (const float*)one, (const int32_t*)one, 0, one, 0, 64, nullptr) == GPTQ_OK);
    EXPECT(gptq_matvec_packed((const uint32_t*)one, 6, 2, 64, 3, (const float*)one, (const int32_t*)one, 4, one, 0, (float*)one, nullptr) == GPTQ_ERR_UNSUPPORTED);
    EXPECT(gptq_matvec_packed((const uint32_t*)one, 6, 0, 64, 3, (const float*)one, (const int32_t*)one, 0, one, 0, (float*)one, nullptr) == GPTQ_OK);

    if (g_failed) { std::printf("%d check(s) failed\n", g_failed); return 1; }
    std::printf("host ABI checks passed under the sanitizers\n");
    return 0;
}
