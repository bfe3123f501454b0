// Step 2: lambda = percdamp * mean(diag H); U = Cholesky((H + lambda I)^-1)^T
// (Section 3, Step 3 and Alg. 1, third statement).
//
// Route: factor H + lambda I = R R^T with R upper triangular -- a Cholesky factorisation that starts at
// the last column and moves backwards -- then invert the triangle, U = R^-1.  (H + lambda I)^-1 =
// R^-T R^-1 = U^T U and the Cholesky factor with positive diagonal is unique, so this U is the
// matrix Alg. 1 asks for, at half the flops of "Cholesky, invert, Cholesky again" and without ever
// forming the explicit inverse.
//
// Two-level blocking (inner 128, outer 1024), everything in place in the upper triangle:
//   factorisation, outer blocks last .. first, inner blocks last .. first:
//     R_bb  = reverse-Cholesky of the 128x128 diagonal block (one workgroup, block in LDS),
//             and its inverse R_bb^-1 kept in the workspace
//     R[0:j0, j0:j1] = H[0:j0, j0:j1] * R_bb^-T             (the panel of R above the block, in place)
//     H[0:j0, outer block columns left of j0] -= R[0:j0, j0:j1] R[.., j0:j1]^T   (rank-128, confined to the outer block)
//     after the outer block: H[0:o0, 0:o0] -= R[0:o0, o] R[0:o0, o]^T   (rank-1024, carries the flops)
//   triangular inverse, outer block columns first .. last:
//     the 1024x1024 diagonal block is inverted in place with rank-128 steps, then
//     U[above, o] = -U[above, above] * (R[above, o] * R_oo^-1)           (K = o0, carries the flops)
#include "common.h"

namespace gptq {

constexpr int NB = 128;
constexpr int DP = NB + 1;      // LDS pitch of the diagonal-block kernels

// One workgroup: mean of the diagonal in float64, lambda in float32, add it to the diagonal.
__global__ __launch_bounds__(1024) void damp_kernel(float* H, int64_t ld, int64_t n, float percdamp, int* info) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 1024) s += (double)H[i * ld + i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    const float lambda = percdamp * (float)(part[0] / (double)n);
    for (int64_t i = threadIdx.x; i < n; i += 1024) H[i * ld + i] += lambda;
    if (threadIdx.x == 0) *info = 0;
}

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---- diagonal block: D = R R^T (R upper, from the last column backwards) and R^-1, 128 x 128 -----------
// Two levels.  A 64 x 64 block is factored and inverted by ONE wavefront entirely in registers: lane i
// owns row i (64 registers, all indices static because the loops are unrolled), and the one value every
// lane needs at a step -- R[k][j] -- sits in lane k and is broadcast with v_readlane.  The 128 x 128
// block combines two of those with 64 x 64 x 64 products on the matrix cores (4 wavefronts, one 32 x 32
// output tile each, operands read from LDS):
//     R22 = rchol(D22), X22 = R22^-1;   R12 = D12 X22^T;   D11 -= R12 R12^T;
//     R11 = rchol(D11), X11 = R11^-1;   X12 = -X11 (R12 X22).

// C[64 x 64] = beta * C + alpha * A[64 x 64] * B, all in LDS with row pitch DP.  B is read as B[k][n] when
// !BT and as B[n][k] when BT.  Called by all 4 wavefronts; wavefront w owns output tile (w / 2, w % 2).
template <bool BT>
__device__ __forceinline__ void mm64(const float* A, const float* B, float* C, float alpha, float beta, int lane, int wave) {
    const int l32 = lane & 31, lhi = lane >> 5;
    const int tm = (wave >> 1) * 32, tn = (wave & 1) * 32;
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll 8
    for (int k = 0; k < 64; k += 2) {
        const float a = A[(tm + l32) * DP + k + lhi];
        const float b = BT ? B[(tn + l32) * DP + k + lhi] : B[(k + lhi) * DP + tn + l32];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float* c = C + (tm + 8 * (i >> 2) + 4 * lhi + (i & 3)) * DP + tn + l32;
        *c = (beta == 0.f) ? alpha * acc[i] : beta * (*c) + alpha * acc[i];
    }
}

// One wavefront: factor the 64 x 64 block at Dm (LDS, pitch DP; upper triangle valid) in place into R and
// write R^-1 to Xm.  Returns the 1-based index of a non-positive pivot inside the block, or 0.
__device__ __forceinline__ int rchol_inv64(float* Dm, float* Xm, int lane) {
    float x[64];
#pragma unroll
    for (int c = 0; c < 64; ++c) x[c] = Dm[lane * DP + c];
    int bad = 0;
#pragma unroll
    for (int j = 63; j >= 0; --j) {
        float dd = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[j]), j));
        if (!(dd > 0.f)) { bad = j + 1; dd = 1.f; }
        const float rj = sqrtf(dd);
        const float inv = 1.0f / rj;
        x[j] = (lane < j) ? x[j] * inv : ((lane == j) ? rj : 0.f);
#pragma unroll
        for (int k = 0; k < j; ++k) {
            const float rkj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[j]), k));
            x[k] = fmaf(-x[j], rkj, x[k]);
        }
    }
#pragma unroll
    for (int c = 0; c < 64; ++c) Dm[lane * DP + c] = x[c];
    // X R = I, column by column: X[i][c] = (delta_ic - sum_{k<c} X[i][k] R[k][c]) / R[c][c]
    float y[64];
#pragma unroll
    for (int c = 0; c < 64; ++c) {
        float s = (lane == c) ? 1.f : 0.f;
#pragma unroll
        for (int k = 0; k < c; ++k) {
            const float rkc = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[c]), k));
            s = fmaf(-y[k], rkc, s);
        }
        const float rcc = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[c]), c));
        y[c] = (lane <= c) ? s / rcc : 0.f;
    }
#pragma unroll
    for (int c = 0; c < 64; ++c) Xm[lane * DP + c] = y[c];
    return bad;
}

// Rows/columns beyond nbk are padded with the identity.  One workgroup of 256 threads.
//   H block  <- R (upper part; strictly lower part of the block zeroed)
//   dinv     <- R^-1 as a dense 128 x 128 block (zeros below the diagonal)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void diag_block_kernel(float* Hblk, int64_t ld, int nbk, float* dinv, int* info, int col_base) {
    extern __shared__ float sm[];
    float* D = sm;                  // [NB][DP]  D, then R
    float* Xs = sm + NB * DP;       // [NB][DP]  R^-1
    float* T = Xs + 64 * DP;        // scratch: the lower-left 64 x 64 block of R^-1, zeroed again at the end
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int q = tid; q < NB * NB; q += 256) {
        const int i = q / NB, k = q % NB;
        float v = (i == k) ? 1.f : 0.f;
        if (i < nbk && k < nbk) v = (k >= i) ? Hblk[(int64_t)i * ld + k] : 0.f;
        D[i * DP + k] = v;
        Xs[i * DP + k] = 0.f;
    }
    __syncthreads();
    float* D11 = D; float* D12 = D + 64; float* D22 = D + 64 * DP + 64;
    float* X11 = Xs; float* X12 = Xs + 64; float* X22 = Xs + 64 * DP + 64;
    int bad = 0;
    if (wave == 0) { bad = rchol_inv64(D22, X22, lane); if (bad) bad += 64; }
    __syncthreads();
    mm64<true>(D12, X22, T, 1.f, 0.f, lane, wave);              // T = D12 X22^T = R12
    __syncthreads();
    for (int q = tid; q < 64 * 64; q += 256) D12[(q >> 6) * DP + (q & 63)] = T[(q >> 6) * DP + (q & 63)];
    __syncthreads();
    mm64<true>(D12, D12, D11, -1.f, 1.f, lane, wave);           // D11 -= R12 R12^T
    mm64<false>(D12, X22, T, 1.f, 0.f, lane, wave);             // T = R12 X22
    __syncthreads();
    if (wave == 0) { const int b1 = rchol_inv64(D11, X11, lane); if (b1) bad = b1; }
    __syncthreads();
    mm64<false>(X11, T, X12, -1.f, 0.f, lane, wave);            // X12 = -X11 (R12 X22)
    if (tid == 0 && bad) atomicCAS(info, 0, col_base + bad);
    __syncthreads();
    for (int q = tid; q < 64 * 64; q += 256) T[(q >> 6) * DP + (q & 63)] = 0.f;
    __syncthreads();
    for (int q = tid; q < NB * NB; q += 256) {
        const int i = q / NB, k = q % NB;
        dinv[q] = Xs[i * DP + k];
        if (i < nbk && k < nbk) Hblk[(int64_t)i * ld + k] = (k >= i) ? D[i * DP + k] : 0.f;
    }
}

// dst[rows x cols] (ld_dst) = src[rows x cols] (ld_src), optionally only the upper triangle of a
// square block (strictly lower part written as zero).
__global__ __launch_bounds__(256) void copy_block_kernel(float* dst, int64_t ld_dst, const float* src, int64_t ld_src,
                                                         int64_t rows, int cols, int upper_square) {
    const int64_t total = rows * cols;
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < total; q += (int64_t)gridDim.x * 256) {
        const int64_t i = q / cols;
        const int k = (int)(q % cols);
        float v = src[i * ld_src + k];
        if (upper_square && k < i) v = 0.f;
        dst[i * ld_dst + k] = v;
    }
}

__global__ __launch_bounds__(256) void zero_lower_kernel(float* H, int64_t ld, int64_t n) {
    const int64_t row = blockIdx.x;
    for (int64_t k = threadIdx.x; k < row; k += 256) H[row * ld + k] = 0.f;
}

}  // namespace gptq

using namespace gptq;

namespace {
constexpr int OB = 1024;     // outer block: rank-1024 updates keep the big GEMMs compute-bound and their tiles long

struct CholWs { float* dinv; float* T; float* dense; size_t total; };
CholWs chol_ws_layout(void* ws, int64_t n) {
    const size_t nblk = (size_t)ceil_div(std::max<int64_t>(n, 1), NB);
    size_t off = 0;
    CholWs l{};
    char* base = static_cast<char*>(ws);
    l.dinv = reinterpret_cast<float*>(base + off);  off += round_up(nblk * NB * NB * sizeof(float), 256);
    l.T = reinterpret_cast<float*>(base + off);     off += round_up((size_t)std::max<int64_t>(n, 1) * OB * sizeof(float), 256);
    l.dense = reinterpret_cast<float*>(base + off); off += (size_t)OB * OB * sizeof(float);
    l.total = off + 256;
    return l;
}
}  // namespace

extern "C" size_t gptq_damp_cholesky_inverse_workspace_bytes(int64_t n) {
    return chol_ws_layout(nullptr, n < 0 ? 0 : n).total;
}

extern "C" int gptq_damp_cholesky_inverse(float* H, int64_t ld, int64_t n, float percdamp,
                                          void* ws, size_t ws_bytes, int* info_dev, void* stream) {
    if (n < 0) return fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: negative size");
    if (!info_dev) return fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: info_dev is null");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) return GPTQ_OK;
    if (!H) return fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: H is null");
    if (ld < n || ld % 4 || !aligned(H, 16))
        return fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: need ld >= n, ld %% 4 == 0 and a 16-byte aligned H");
    if (!(percdamp >= 0.f)) return fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: percdamp must be >= 0");
    if (!ws || !aligned(ws, 256) || ws_bytes < gptq_damp_cholesky_inverse_workspace_bytes(n))
        return fail(GPTQ_ERR_WORKSPACE, "damp_cholesky_inverse: workspace missing, misaligned or too small");

    const CholWs w = chol_ws_layout(ws, n);
    float* dinv = w.dinv;
    constexpr size_t diag_lds = 2 * NB * DP * sizeof(float);
    GPTQ_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(diag_block_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)diag_lds));

    hipLaunchKernelGGL(damp_kernel, dim3(1), dim3(1024), 0, s, H, ld, n, percdamp, info_dev);
    GPTQ_LAUNCH_CHECK();

    auto gemm_on = [&](hipStream_t st, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                       float alpha, bool nk, bool overwrite, bool upper, int64_t crow0, int64_t ccol0, bool atri) -> int {
        GemmF32 g{};
        g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
        g.b_is_nk = nk; g.overwrite = overwrite; g.upper_only = upper; g.crow0 = crow0; g.ccol0 = ccol0; g.a_upper_tri = atri;
        return launch_gemm_f32(g, st);
    };
    auto gemm = [&](const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                    float alpha, bool nk, bool overwrite, bool upper, int64_t crow0, int64_t ccol0, bool atri) -> int {
        return gemm_on(s, A, lda, B, ldb, C, ldc, M, N, K, alpha, nk, overwrite, upper, crow0, ccol0, atri);
    };
    const int64_t nouter = ceil_div(n, OB);
    Lookahead* la = nullptr;
    if (int rc = lookahead_get(&la)) return rc;
    hipStream_t s2 = la->stream;

    // ---- H + lambda I = R R^T, from the last column backwards.  Two levels: inside an outer block of
    //      1024 columns the rank-128 updates touch only that block's columns; the rest of the matrix gets
    //      one rank-1024 update per outer block.
    hipEvent_t rest_done = nullptr;         // the helper stream's last trailing update, if one is pending
    for (int64_t o = nouter - 1; o >= 0; --o) {
        const int64_t o0 = o * OB, o1 = std::min<int64_t>(o0 + OB, n);
        for (int64_t j0 = (ceil_div(o1 - o0, NB) - 1) * NB + o0; j0 >= o0; j0 -= NB) {
            const int nbk = (int)std::min<int64_t>(NB, n - j0);
            float* dinv_b = dinv + (j0 / NB) * NB * NB;
            hipLaunchKernelGGL(diag_block_kernel, dim3(1), dim3(256), diag_lds, s, H + j0 * ld + j0, ld, nbk, dinv_b, info_dev, (int)j0);
            GPTQ_LAUNCH_CHECK();
            if (j0 == 0) break;
            // R[0:j0, j0:j1] = H[0:j0, j0:j1] * R_bb^-T, the panel of R above the block.  In place: there is a
            // single tile column, and a workgroup reads all of its own rows before it writes them.
            int rc = gemm(H + j0, ld, dinv_b, NB, H + j0, ld, j0, nbk, nbk, 1.f, true, true, false, 0, 0, false);
            if (rc) return rc;
            // H[0:j0, o0:j0] -= R[0:j0, j0:j1] * R[o0:j0, j0:j1]^T  (columns of this outer block only; tiles below the
            // diagonal skipped).  Right-looking: many short tiles, which keeps this serial chain short; a left-looking
            // product per inner block (one tile column, K up to 896) measured slower on mid-size matrices.
            if (j0 > o0) {
                rc = gemm(H + j0, ld, H + o0 * ld + j0, ld, H + o0, ld, j0, j0 - o0, nbk, -1.f, true, false, true, 0, o0, false);
                if (rc) return rc;
            }
        }
        // H[0:o0, 0:o0] -= R[0:o0, o0:o1] * R[0:o0, o0:o1]^T  (rank-1024, upper tiles), with look-ahead:
        // the columns [p0, o0) of the next outer block are updated first, on the caller's stream, which then
        // goes on to factor that block (short, serial kernels); the rest, H[0:p0, 0:p0], is updated on the
        // helper stream meanwhile.  The two parts and the next block's factorisation write disjoint regions;
        // the next block's own column update waits for the helper's, which wrote the same region.
        if (o0 > 0) {
            const int64_t p0 = o0 - OB;                  // outer blocks start at multiples of OB
            hipEvent_t factored = la->event();
            GPTQ_HIP_CHECK(hipEventRecord(factored, s));
            if (rest_done) GPTQ_HIP_CHECK(hipStreamWaitEvent(s, rest_done, 0));
            int rc = gemm(H + o0, ld, H + p0 * ld + o0, ld, H + p0, ld, o0, o0 - p0, o1 - o0, -1.f, true, false, true, 0, p0, false);
            if (rc) return rc;
            if (p0 > 0) {
                GPTQ_HIP_CHECK(hipStreamWaitEvent(s2, factored, 0));
                rc = gemm_on(s2, H + o0, ld, H + o0, ld, H, ld, p0, p0, o1 - o0, -1.f, true, false, true, 0, 0, false);
                if (rc) return rc;
                rest_done = la->event();
                GPTQ_HIP_CHECK(hipEventRecord(rest_done, s2));
            } else {
                rest_done = nullptr;
            }
        }
    }

    // The triangular GEMMs below skip the K range left of a tile's first row and rely on zeros below the
    // diagonal inside the tile's own rows, so clear the strictly lower triangle first (it holds the input's
    // lower half and the below-diagonal parts of straddling update tiles); nothing writes there afterwards.
    hipLaunchKernelGGL(zero_lower_kernel, dim3((unsigned)n), dim3(256), 0, s, H, ld, n);
    GPTQ_LAUNCH_CHECK();
    {
        hipEvent_t cleared = la->event();
        GPTQ_HIP_CHECK(hipEventRecord(cleared, s));
        GPTQ_HIP_CHECK(hipStreamWaitEvent(s2, cleared, 0));
    }

    // ---- U = R^-1 in place, one outer block column at a time (left to right):
    //      invert the 1024 x 1024 diagonal block in place with rank-128 steps, then
    //      U[above, o] = -U[above, above] * (R[above, o] * R_oo^-1), a long-K GEMM against the finished part.
    //      The in-block inversions touch nothing but their own diagonal block, so they all run ahead on the
    //      helper stream while the caller's stream carries the long GEMMs, each waiting for its block's event.
    for (int64_t o = 0; o < nouter; ++o) {
        const int64_t o0 = o * OB, o1 = std::min<int64_t>(o0 + OB, n);
        for (int64_t j0 = o0; j0 < o1; j0 += NB) {
            const int nbk = (int)std::min<int64_t>(NB, n - j0);
            const int64_t j1 = j0 + nbk;
            const float* dinv_b = dinv + (j0 / NB) * NB * NB;
            if (j1 < o1) {
                // R[b, right] = -R_bb^-1 * R[b, right].  In place: a workgroup reads its own 128 columns of all
                // (<= 128) rows through LDS before its epilogue writes them, and there is a single tile row.
                int rc = gemm_on(s2, dinv_b, NB, H + j0 * ld + j1, ld, H + j0 * ld + j1, ld, nbk, o1 - j1, nbk, -1.f, false, true, false, 0, 0, false);
                if (rc) return rc;
                if (j0 > o0) {
                    rc = gemm_on(s2, H + o0 * ld + j0, ld, H + j0 * ld + j1, ld, H + o0 * ld + j1, ld, j0 - o0, o1 - j1, nbk, 1.f, false, false, false, 0, 0, false);
                    if (rc) return rc;
                }
            }
            if (j0 > o0) {
                // R[above-in-block, b] = R[above-in-block, b] * R_bb^-1.  In place: a single tile column, each
                // workgroup reads all of its own rows before writing them.
                const int rc = gemm_on(s2, H + o0 * ld + j0, ld, dinv_b, NB, H + o0 * ld + j0, ld, j0 - o0, nbk, nbk, 1.f, false, true, false, 0, 0, false);
                if (rc) return rc;
            }
            hipLaunchKernelGGL(copy_block_kernel, dim3(64), dim3(256), 0, s2, H + j0 * ld + j0, ld, dinv_b, (int64_t)NB, (int64_t)nbk, nbk, 1);
            GPTQ_LAUNCH_CHECK();
        }
        {
            hipEvent_t inverted = la->event();
            GPTQ_HIP_CHECK(hipEventRecord(inverted, s2));
            GPTQ_HIP_CHECK(hipStreamWaitEvent(s, inverted, 0));
        }
        if (o0 > 0) {
            const int ow = (int)(o1 - o0);
            // dense copy of the inverted diagonal block with an explicit zero lower triangle
            hipLaunchKernelGGL(copy_block_kernel, dim3(256), dim3(256), 0, s, w.dense, (int64_t)OB, (const float*)(H + o0 * ld + o0), ld, (int64_t)ow, ow, 1);
            GPTQ_LAUNCH_CHECK();
            int rc = gemm(H + o0, ld, w.dense, OB, w.T, OB, o0, ow, ow, 1.f, false, true, false, 0, 0, false);
            if (rc) return rc;
            rc = gemm(H, ld, w.T, OB, H + o0, ld, o0, ow, o0, -1.f, false, true, false, 0, 0, true);
            if (rc) return rc;
        }
    }
    return GPTQ_OK;
}

extern "C" int gptq_check_info(const int* info_dev, int* host_info, void* stream) {
    if (!info_dev) return fail(GPTQ_ERR_INVALID_ARG, "check_info: info_dev is null");
    hipStream_t s = static_cast<hipStream_t>(stream);
    int v = 0;
    GPTQ_HIP_CHECK(hipMemcpyAsync(&v, info_dev, sizeof(int), hipMemcpyDeviceToHost, s));
    GPTQ_HIP_CHECK(hipStreamSynchronize(s));
    if (host_info) *host_info = v;
    if (v != 0) return fail(GPTQ_ERR_NOT_POSDEF, "pivot of column %d (1-based) was not positive", v);
    return GPTQ_OK;
}
