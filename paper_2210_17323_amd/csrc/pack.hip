// Step 4: dense bit packing of 2/3/4-bit codes (the paper stores 3-bit weights densely,
// Section 4 "Practical Speedups", without printing a layout; this one is ours).
//
// Per row, code k occupies bits [k*b, (k+1)*b) of a little-endian stream of uint32 words.
// 32 codes always fill exactly b words, so one thread turns 32 consecutive codes (two 16-byte
// loads) into b consecutive words; neighbouring threads read and write neighbouring addresses.
#include "common.h"

namespace gptq {

template <int BITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* codes, int64_t ldc, int64_t r, int64_t n,
                                                   uint32_t* out, int64_t ldo, int64_t groups_per_row, int vec_ok) {
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= r * groups_per_row) return;
    const int64_t row = gid / groups_per_row, grp = gid % groups_per_row;
    const int64_t k0 = grp * 32;
    const uint8_t* src = codes + row * ldc + k0;
    uint8_t c[32];
    if (vec_ok && k0 + 32 <= n) {
        const uint4 a = *reinterpret_cast<const uint4*>(src);
        const uint4 b = *reinterpret_cast<const uint4*>(src + 16);
        const uint32_t wds[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 32; ++i) c[i] = (uint8_t)(wds[i >> 2] >> (8 * (i & 3)));
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) c[i] = (k0 + i < n) ? src[i] : (uint8_t)0;
    }
    uint32_t w[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) w[i] = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const uint32_t v = c[i] & ((1u << BITS) - 1u);
        const int pos = i * BITS, wi = pos >> 5, off = pos & 31;
        w[wi] |= v << off;
        if (off + BITS > 32) w[wi + 1] |= v >> (32 - off);
    }
    const int64_t words_per_row = (n * BITS + 31) / 32;
    uint32_t* dst = out + row * ldo + grp * BITS;
#pragma unroll
    for (int i = 0; i < BITS; ++i)
        if (grp * BITS + i < words_per_row) dst[i] = w[i];
}

template <int BITS>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* words, int64_t ldw, int64_t r, int64_t n,
                                                     uint8_t* codes, int64_t ldc, int64_t groups_per_row) {
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= r * groups_per_row) return;
    const int64_t row = gid / groups_per_row, grp = gid % groups_per_row;
    const int64_t words_per_row = (n * BITS + 31) / 32;
    uint32_t w[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) w[i] = (grp * BITS + i < words_per_row) ? words[row * ldw + grp * BITS + i] : 0u;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int pos = i * BITS, wi = pos >> 5, off = pos & 31;
        uint32_t v = w[wi] >> off;
        if (off + BITS > 32) v |= w[wi + 1] << (32 - off);
        const int64_t k = grp * 32 + i;
        if (k < n) codes[row * ldc + k] = (uint8_t)(v & ((1u << BITS) - 1u));
    }
}

}  // namespace gptq

using namespace gptq;

static int check_pack_args(const void* a, const void* b, int64_t r, int64_t n, int bits, int64_t ld_codes, int64_t ld_words, const char* who) {
    if (r < 0 || n < 0) return fail(GPTQ_ERR_INVALID_ARG, "%s: negative size", who);
    if (bits < 2 || bits > 4) return fail(GPTQ_ERR_INVALID_ARG, "%s: bits must be 2, 3 or 4 (got %d)", who, bits);
    if (r == 0 || n == 0) return GPTQ_OK;
    if (!a || !b) return fail(GPTQ_ERR_INVALID_ARG, "%s: null pointer", who);
    if (ld_codes < n) return fail(GPTQ_ERR_INVALID_ARG, "%s: ldc < n", who);
    if (ld_words < (n * bits + 31) / 32) return fail(GPTQ_ERR_INVALID_ARG, "%s: word pitch smaller than ceil(n*bits/32)", who);
    if (r * ((n + 31) / 32) > (int64_t)0x7fffffff * 256) return fail(GPTQ_ERR_UNSUPPORTED, "%s: too large", who);
    return -1;
}

extern "C" int gptq_pack(const uint8_t* codes, int64_t ldc, int64_t r, int64_t n, int bits,
                         uint32_t* out, int64_t ld_out, void* stream) {
    const int rc = check_pack_args(codes, out, r, n, bits, ldc, ld_out, "pack");
    if (rc >= 0) return rc;
    const int64_t gpr = (n + 31) / 32;
    const unsigned blocks = (unsigned)ceil_div(r * gpr, 256);
    const int vec_ok = aligned(codes, 16) && (ldc % 16 == 0);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bits == 2) hipLaunchKernelGGL(pack_kernel<2>, dim3(blocks), dim3(256), 0, s, codes, ldc, r, n, out, ld_out, gpr, vec_ok);
    else if (bits == 3) hipLaunchKernelGGL(pack_kernel<3>, dim3(blocks), dim3(256), 0, s, codes, ldc, r, n, out, ld_out, gpr, vec_ok);
    else hipLaunchKernelGGL(pack_kernel<4>, dim3(blocks), dim3(256), 0, s, codes, ldc, r, n, out, ld_out, gpr, vec_ok);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

extern "C" int gptq_unpack(const uint32_t* words, int64_t ld_words, int64_t r, int64_t n, int bits,
                           uint8_t* codes, int64_t ldc, void* stream) {
    const int rc = check_pack_args(codes, words, r, n, bits, ldc, ld_words, "unpack");
    if (rc >= 0) return rc;
    const int64_t gpr = (n + 31) / 32;
    const unsigned blocks = (unsigned)ceil_div(r * gpr, 256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bits == 2) hipLaunchKernelGGL(unpack_kernel<2>, dim3(blocks), dim3(256), 0, s, words, ld_words, r, n, codes, ldc, gpr);
    else if (bits == 3) hipLaunchKernelGGL(unpack_kernel<3>, dim3(blocks), dim3(256), 0, s, words, ld_words, r, n, codes, ldc, gpr);
    else hipLaunchKernelGGL(unpack_kernel<4>, dim3(blocks), dim3(256), 0, s, words, ld_words, r, n, codes, ldc, gpr);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}
