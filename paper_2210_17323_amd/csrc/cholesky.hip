// Step 2: lambda = percdamp * mean(diag H); U = Cholesky((H + lambda I)^-1)^T
// (Section 3, Step 3 and Alg. 1, third statement).
//
// Route: factor H + lambda I = R R^T with R upper triangular -- a Cholesky factorisation that starts at
// the last column and moves backwards -- then invert the triangle, U = R^-1.  (H + lambda I)^-1 =
// R^-T R^-1 = U^T U and the Cholesky factor with positive diagonal is unique, so this U is the
// matrix Alg. 1 asks for, at half the flops of "Cholesky, invert, Cholesky again" and without ever
// forming the explicit inverse.
//
// Two-level blocking (inner blocks of 128 columns, outer blocks of 1024), result in place in the upper triangle.
//
// Factorisation, outer blocks o last .. first, inner blocks b last .. first:
//     R_bb = reverse-Cholesky of the 128 x 128 diagonal block (one workgroup, block in LDS), R_bb^-1 kept
//     R[0:j0, b] = H[0:j0, b] R_bb^-T                                  (the panel of R above the block, in place)
//     H[0:j0, outer block's columns left of b] -= R[0:j0, b] R[.., b]^T   (rank 128, confined to the outer block)
//   after the outer block: H[0:o0, 0:o0] -= R[0:o0, o] R[0:o0, o]^T   (rank 1024, carries the flops)
//   one step behind, on a stream of its own (only when the inverse is wanted): the row blocks of U_oo = R_oo^-1,
//     U[b, right] = -R_bb^-1 (R[b, right] U[right, right]), kept dense for the inverse.
//
// Triangular inverse (right-looking, outer block columns k first .. last), with the U_kk kept from the factorisation:
//     T = -U_kk R[k, right of k] ;  U[above k, right of k] += U[above k, k] T ;  row block k <- T
//     U[above k, k] <- U[above k, k] U_kk ;  diagonal block <- U_kk
// Every long product has K = 1024 and an output of (rows above) x (columns to the right): many tiles at every k.
#include "common.h"

#include <mutex>

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
// Two levels.  A 32 x 32 block is factored and inverted by ONE wavefront in registers: lane i owns row i
// (32 registers, all indices static because the loops are unrolled); the one thing every lane needs at a
// step -- column j of the block -- goes through a small LDS buffer that all lanes read back with uniform
// (broadcast) addresses.  The 128 x 128 block combines four of those with 32 x 32 x 32 products on the
// matrix cores (4 wavefronts, one output tile each, operands read from LDS).  With block indices
// b = 3 .. 0 and R_bc, X_bc the tiles of R and of X = R^-1:
//     step b, part 1:  wavefront 0: R_bb = rchol(D_bb), X_bb = R_bb^-1
//                      the others:  S_bc' = sum_{b < c <= c'} R_bc X_cc'  for c' > b   (needs nothing of part 1)
//     step b, part 2:  R_ab = D_ab X_bb^T for a < b;   X_bc' = -X_bb S_bc' for c' > b
//     step b, part 3:  D_aa' -= R_ab R_a'b^T for a <= a' < b

// acc += A[32 x 32] * B, operands in LDS with row pitch DP.  B is read as B[k][n] when !BT and as B[n][k]
// when BT.  One wavefront.
template <bool BT>
__device__ __forceinline__ void mma32(floatx16& acc, const float* A, const float* B, int lane) {
    const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
    for (int k = 0; k < 32; k += 2) {
        const float a = A[l32 * DP + k + lhi];
        const float b = BT ? B[l32 * DP + k + lhi] : B[(k + lhi) * DP + l32];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
}

// C[32 x 32] = beta * C + alpha * acc (C in LDS, pitch DP).  One wavefront.
__device__ __forceinline__ void store32(float* C, const floatx16& acc, float alpha, float beta, int lane) {
    const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float* c = C + (8 * (i >> 2) + 4 * lhi + (i & 3)) * DP + l32;
        *c = (beta == 0.f) ? alpha * acc[i] : beta * (*c) + alpha * acc[i];
    }
}

__device__ __forceinline__ floatx16 zero16() {
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    return acc;
}

// One wavefront: factor the 32 x 32 block at Dm (LDS, pitch DP; upper triangle valid) in place into R and
// write R^-1 to Xm.  Ct is a 32 x 64 LDS buffer that receives the columns: Ct[j][k], k < 32, = the
// finished, not yet scaled column j of the block, i.e. R[k][j] * R[j][j].  Lanes 32 .. 63 mirror lanes
// 0 .. 31; their copies of a column land in the unused half of its row of Ct, nothing else is stored.  Below the diagonal Dm is left with values that mean nothing (nobody reads them: they
// only ever combine with each other); Xm is a clean upper triangle.  Returns the 1-based index of the
// first non-positive pivot met, or 0.
__device__ __forceinline__ int rchol_inv32(float* Dm, float* Xm, float* Ct, int lane) {
    int row = lane & 31;
    asm volatile("" : "+v"(row));      // keeps the lane tests below next to their uses instead of hoisted and spilled
    const bool owner = lane < 32;
    float x[32], rinv[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) x[c] = Dm[row * DP + c];
    int bad = 0;
    Ct[31 * 64 + lane] = x[31];
#pragma unroll
    for (int j = 31; j >= 0; --j) {
        // column j is final: every lane reads all of it.  R[k][j] = col[k] / r, R[j][j] = r = sqrt(col[j]).
        float col[32];
#pragma unroll
        for (int k = 0; k <= j; ++k) col[k] = Ct[j * 64 + k];
        float dd = col[j];
        if (!(dd > 0.f)) { if (!bad) bad = j + 1; dd = 1.f; }
        float inv = __frsqrt_rn(dd);
        inv = inv * fmaf(-0.5f * dd * inv, inv, 1.5f);       // one Newton step: 1 / sqrt(dd) to an ulp
        rinv[j] = inv;
        const float u = x[j] * inv * inv;                     // R[row][j] / r
        x[j] *= inv;                                          // row j: dd / sqrt(dd) = r
        // x[k] -= R[row][j] R[k][j]; the column needed next goes out first so that its round trip through
        // LDS overlaps the rest of the update
#pragma unroll
        for (int k = j - 1; k >= 0; --k) {
            x[k] = fmaf(-u, col[k], x[k]);
            if (k == j - 1) Ct[(j - 1) * 64 + lane] = x[k];
        }
    }
    if (owner) {
#pragma unroll
        for (int c = 0; c < 32; ++c) Dm[row * DP + c] = x[c];
    }
    // X R = I, column by column: X[i][c] = (delta_ic - sum_{k<c} X[i][k] R[k][c]) / R[c][c].  Rows below
    // the diagonal come out as exact zeros: every term of their sums is one.
    float y[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < c; ++k) s = fmaf(y[k], Ct[c * 64 + k], s);
        const float d = (row == c) ? rinv[c] : 0.f;
        y[c] = fmaf(-rinv[c] * rinv[c], s, d);
    }
    if (owner) {
#pragma unroll
        for (int c = 0; c < 32; ++c) Xm[row * DP + c] = y[c];
    }
    return bad;
}

// Rows/columns beyond nbk are padded with the identity.  One workgroup of 256 threads.
//   H block  <- R (upper part; strictly lower part of the block zeroed)
//   dinv     <- R^-1 as a dense 128 x 128 block (zeros below the diagonal)
__global__ __launch_bounds__(256)
void diag_block_kernel(float* Hblk, int64_t ld, int nbk, float* dinv, int* info, int col_base) {
    extern __shared__ __align__(16) float sm[];
    float* Ct = sm;                 // [32][64]  columns of the block being factored
    float* D = sm + 32 * 64;        // [NB][DP]  D, then R
    float* Xs = D + NB * DP;        // [NB][DP]  R^-1 (tiles right of the diagonal hold S until part 2)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // 16 independent 16-byte loads per thread, all in flight together: the block arrives in one round trip
    float4 in[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int q = tid + 256 * t, i = q >> 5, k = (q & 31) * 4;
        const float* src = Hblk + (int64_t)i * ld + k;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < nbk && k + 4 <= nbk) v = *reinterpret_cast<const float4*>(src);
        else if (i < nbk && k < nbk) { v.x = src[0]; if (k + 1 < nbk) v.y = src[1]; if (k + 2 < nbk) v.z = src[2]; }
        in[t] = v;
    }
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int q = tid + 256 * t, i = q >> 5, k = (q & 31) * 4;
        const float e[4] = {in[t].x, in[t].y, in[t].z, in[t].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int kc = k + c;
            const bool inside = i < nbk && kc < nbk;
            D[i * DP + kc] = inside ? (kc >= i ? e[c] : 0.f) : (i == kc ? 1.f : 0.f);
            Xs[i * DP + kc] = 0.f;
        }
    }
    __syncthreads();
    auto tile = [](float* base, int a, int c) { return base + a * 32 * DP + c * 32; };
    int bad = 0;
#pragma unroll 1
    for (int b = 3; b >= 0; --b) {
        if (wave == 0) {
            const int b1 = rchol_inv32(tile(D, b, b), tile(Xs, b, b), Ct, lane);
            if (b1 && !bad) bad = b * 32 + b1;
        } else if (b + wave <= 3) {
            const int cp = b + wave;                            // S_b,cp = sum_{b < c <= cp} R_bc X_c,cp
            floatx16 acc = zero16();
            for (int c = b + 1; c <= cp; ++c) mma32<false>(acc, tile(D, b, c), tile(Xs, c, cp), lane);
            store32(tile(Xs, b, cp), acc, 1.f, 0.f, lane);
        }
        __syncthreads();
        if (wave < 3) {
            floatx16 acc = zero16();
            if (wave < b) {                                     // R_ab = D_ab X_bb^T, in place
                mma32<true>(acc, tile(D, wave, b), tile(Xs, b, b), lane);
                store32(tile(D, wave, b), acc, 1.f, 0.f, lane);
            } else {                                            // X_b,cp = -X_bb S_b,cp, in place
                const int cp = wave + 1;
                mma32<false>(acc, tile(Xs, b, b), tile(Xs, b, cp), lane);
                store32(tile(Xs, b, cp), acc, -1.f, 0.f, lane);
            }
        }
        __syncthreads();
        // D_aa' -= R_ab R_a'b^T for a <= a' < b: b (b + 1) / 2 tiles dealt over the wavefronts
        for (int t = wave; t < b * (b + 1) / 2; t += 4) {
            int a = 0, rest = t;                                // tile number t in the order (0,0) .. (0,b-1) (1,1) ..
            while (rest >= b - a) { rest -= b - a; ++a; }
            const int ap = a + rest;
            floatx16 acc = zero16();
            mma32<true>(acc, tile(D, a, b), tile(D, ap, b), lane);
            store32(tile(D, a, ap), acc, -1.f, 1.f, lane);
        }
        __syncthreads();
    }
    if (tid == 0 && bad) atomicCAS(info, 0, col_base + bad);
#pragma unroll 4
    for (int t = 0; t < 16; ++t) {
        const int q = tid + 256 * t, i = q >> 5, k = (q & 31) * 4;
        float4 xv, rv;
        xv.x = Xs[i * DP + k]; xv.y = Xs[i * DP + k + 1]; xv.z = Xs[i * DP + k + 2]; xv.w = Xs[i * DP + k + 3];
        rv.x = (k >= i) ? D[i * DP + k] : 0.f;         rv.y = (k + 1 >= i) ? D[i * DP + k + 1] : 0.f;
        rv.z = (k + 2 >= i) ? D[i * DP + k + 2] : 0.f; rv.w = (k + 3 >= i) ? D[i * DP + k + 3] : 0.f;
        reinterpret_cast<float4*>(dinv)[q] = xv;
        float* dst = Hblk + (int64_t)i * ld + k;
        if (i < nbk && k + 4 <= nbk) *reinterpret_cast<float4*>(dst) = rv;
        else if (i < nbk && k < nbk) { dst[0] = rv.x; if (k + 1 < nbk) dst[1] = rv.y; if (k + 2 < nbk) dst[2] = rv.z; }
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

// dst[rows x cols] = src[rows x cols]; both 16-byte aligned with leading dimensions and cols that are multiples of 4
__global__ __launch_bounds__(256) void copy2d_kernel(float* dst, int64_t ld_dst, const float* src, int64_t ld_src, int64_t rows, int64_t cols4) {
    const int64_t total = rows * cols4;
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < total; q += (int64_t)gridDim.x * 256) {
        const int64_t i = q / cols4, c = q - i * cols4;
        reinterpret_cast<float4*>(dst + i * ld_dst)[c] = reinterpret_cast<const float4*>(src + i * ld_src)[c];
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float4* p, int64_t count4) {
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < count4; q += (int64_t)gridDim.x * 256)
        p[q] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ __launch_bounds__(256) void zero_lower_kernel(float* H, int64_t ld, int64_t n) {
    const int64_t row = blockIdx.x;
    for (int64_t k = threadIdx.x; k < row; k += 256) H[row * ld + k] = 0.f;
}

}  // namespace gptq

using namespace gptq;

namespace {
constexpr int OB = 1024;     // outer block: rank-1024 updates keep the big GEMMs compute-bound and their tiles long
static_assert(OB == SPLIT_K, "the split products take exactly one outer block as K");
// A rank-1024 update goes through the split-operand kernel (bf16 matrix cores, 256 x 256 tiles) when its tiles fill the
// chip well (split_pays): the strip of the next outer block has 4 tile columns, the square rest t (t + 1) / 2 tiles.

struct CholWs { float* dinv; float* T; float* T2; int64_t ld2; float* Uoo; float* tmp; unsigned char* planes; unsigned char* planes2; size_t total; };
CholWs chol_ws_layout(void* ws, int64_t n, bool with_split = true) {
    const size_t n1 = (size_t)std::max<int64_t>(n, 1);
    const size_t nblk = (size_t)ceil_div((int64_t)n1, NB), nouter = (size_t)ceil_div((int64_t)n1, OB);
    size_t off = 0;
    CholWs l{};
    // with ws == nullptr only the total is wanted: no pointer is formed (arithmetic on a null pointer is undefined)
    uintptr_t base = reinterpret_cast<uintptr_t>(ws);
    auto at = [&](size_t bytes) { const size_t o = off; off += round_up(bytes, 256); return ws ? reinterpret_cast<void*>(base + o) : nullptr; };
    l.ld2 = (int64_t)round_up(n1, 4);
    l.dinv = static_cast<float*>(at(nblk * NB * NB * sizeof(float)));        // R_bb^-1, dense
    l.T = static_cast<float*>(at(n1 * OB * sizeof(float)));                  // a column panel [n x 1024]
    l.T2 = static_cast<float*>(at((size_t)OB * l.ld2 * sizeof(float)));      // a row panel [1024 x n]
    l.Uoo = static_cast<float*>(at(nouter * OB * OB * sizeof(float)));       // U_oo of every outer block, dense
    l.tmp = static_cast<float*>(at((size_t)NB * OB * sizeof(float)));        // one row block of a product
    if (with_split && (int64_t)n1 >= 2 * OB) {                               // split products: bf16 pieces of a column panel
        l.planes = static_cast<unsigned char*>(at(split_planes_bytes((int64_t)n1)));
        l.planes2 = static_cast<unsigned char*>(at(split_planes_bytes((int64_t)n1)));      // ... and of a row block (the inverse)
    }
    l.total = off + 256;
    return l;
}
}  // namespace

extern "C" size_t gptq_damp_cholesky_inverse_workspace_bytes(int64_t n) {
    return chol_ws_layout(nullptr, n < 0 ? 0 : n).total;
}

// Host-side checks shared by the entry points; 1 = nothing to do (n == 0).
static int chol_check_args(const float* H, int64_t ld, int64_t n, float percdamp, const int* info_dev, int* rc) {
    *rc = GPTQ_OK;
    if (n < 0) { *rc = fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: negative size"); return 1; }
    if (!info_dev) { *rc = fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: info_dev is null"); return 1; }
    if (n == 0) return 1;
    if (!H) { *rc = fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: H is null"); return 1; }
    if (ld < n || ld % 4 || !aligned(H, 16)) {
        *rc = fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: need ld >= n, ld %% 4 == 0 and a 16-byte aligned H");
        return 1;
    }
    if (!(percdamp >= 0.f)) { *rc = fail(GPTQ_ERR_INVALID_ARG, "damp_cholesky_inverse: percdamp must be >= 0"); return 1; }
    return 0;
}

// The whole of step 2 on validated arguments.  `ws` holds chol_ws_layout(n).total bytes; nothing in it has to be
// initialised (every region is written in this call before it is read).  lookahead = false keeps all work on `s`
// (the host code below enqueues in an order that respects every dependence, so one stream is always valid).
// want_inverse = false stops after the factorisation: H holds R (upper triangular, zeros below) with H + lambda I = R R^T.
static int chol_run(float* H, int64_t ld, int64_t n, float percdamp, void* ws, int* info_dev, hipStream_t s, bool lookahead,
                    bool want_inverse = true, bool with_split = true) {
    const CholWs w = chol_ws_layout(ws, n, with_split);
    float* dinv = w.dinv;
    constexpr size_t diag_lds = (2 * NB * DP + 32 * 64) * sizeof(float);
    GPTQ_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(diag_block_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)diag_lds));

    hipLaunchKernelGGL(damp_kernel, dim3(1), dim3(1024), 0, s, H, ld, n, percdamp, info_dev);
    GPTQ_LAUNCH_CHECK();

    // C (+)= alpha A op(B) on stream st
    struct Opt { bool nk = false, overwrite = false, upper = false, atri = false, btri = false; int64_t crow0 = 0, ccol0 = 0; int cap = 0; };
    auto gemm_on = [&](hipStream_t st, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                       int64_t M, int64_t N, int64_t K, float alpha, const Opt& o) -> int {
        GemmF32 g{};
        g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
        g.b_is_nk = o.nk; g.overwrite = o.overwrite; g.upper_only = o.upper; g.crow0 = o.crow0; g.ccol0 = o.ccol0;
        g.a_upper_tri = o.atri; g.b_upper_tri = o.btri; g.max_workgroups = o.cap;
        return launch_gemm_f32(g, st);
    };
    auto copy2d = [&](hipStream_t st, float* dst, int64_t ld_dst, const float* src, int64_t ld_src, int64_t rows, int64_t cols) -> int {
        if (rows <= 0 || cols <= 0) return GPTQ_OK;
        if (cols % 4 == 0 && ld_dst % 4 == 0 && ld_src % 4 == 0 && aligned(dst, 16) && aligned(src, 16)) {
            const int64_t total4 = rows * (cols / 4);
            hipLaunchKernelGGL(copy2d_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(total4, 256), 2048)), dim3(256), 0, st, dst, ld_dst, src, ld_src, rows, cols / 4);
        } else {
            hipLaunchKernelGGL(copy_block_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(rows * cols, 256), 2048)), dim3(256), 0, st, dst, ld_dst, src, ld_src, rows, (int)cols, 0);
        }
        GPTQ_LAUNCH_CHECK();
        return GPTQ_OK;
    };
    const int64_t nouter = ceil_div(n, OB);
    TwoStreams ts;
    if (int rc = ts.open(s, lookahead)) return rc;
    hipStream_t s2 = ts.side;       // long products: panels through U_oo and rank-1024 updates
    hipStream_t s3 = ts.side2;      // (joined below; carries nothing here)
    hipStream_t s4 = ts.side3;      // trails the factorisation's chain: the rows of U_oo

    // ---- H + lambda I = R R^T, from the last column backwards.  Two levels: inside an outer block of 1024 columns the
    //      rank-128 updates touch only that block's columns; the rest of the matrix gets one rank-1024 update per block.
    hipEvent_t rest_done = nullptr;     // s2: the last rank-1024 update, if one is pending
    for (int64_t o = nouter - 1; o >= 0; --o) {
        const int64_t o0 = o * OB, o1 = std::min<int64_t>(o0 + OB, n), ow = o1 - o0;
        float* Ublk = w.Uoo + o * (int64_t)OB * OB;      // U_oo = R_oo^-1 [ow x ow], leading dimension OB, for the inverse
        if (want_inverse) {                              // zeros below the diagonal are relied on by the products that read it
            hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, s4, reinterpret_cast<float4*>(Ublk), (int64_t)OB * OB / 4);
            GPTQ_LAUNCH_CHECK();
        }
        for (int64_t j0 = (ceil_div(ow, NB) - 1) * NB + o0; j0 >= o0; j0 -= NB) {
            const int nbk = (int)std::min<int64_t>(NB, n - j0);
            const int64_t j1 = j0 + nbk;
            float* dinv_b = dinv + (j0 / NB) * NB * NB;
            hipLaunchKernelGGL(diag_block_kernel, dim3(1), dim3(256), diag_lds, s, H + j0 * ld + j0, ld, nbk, dinv_b, info_dev, (int)j0);
            GPTQ_LAUNCH_CHECK();
            if (j0 > 0) {
                // R[0:j0, b] = H[0:j0, b] R_bb^-T, the panel of R above the block.  In place: there is a single tile column,
                // and a workgroup reads all of its own rows before it writes them.
                Opt po; po.nk = true; po.overwrite = true;
                if (int rc = gemm_on(s, H + j0, ld, dinv_b, NB, H + j0, ld, j0, nbk, nbk, 1.f, po)) return rc;
            }
            if (want_inverse) {
                // One step behind, on its own stream: the row block of U_oo,
                // U[b, b] = R_bb^-1,  U[b, right] = -R_bb^-1 (R[b, right] U[right, right])  (U[right, right] upper triangular)
                hipEvent_t step = nullptr;
                if (int rc = ts.mark(s, &step)) return rc;
                if (int rc = ts.wait(s4, step)) return rc;
                const int64_t d = j0 - o0;               // position of the row block inside U_oo
                hipLaunchKernelGGL(copy_block_kernel, dim3(64), dim3(256), 0, s4, Ublk + d * OB + d, (int64_t)OB, (const float*)dinv_b, (int64_t)NB, (int64_t)nbk, nbk, 1);
                GPTQ_LAUNCH_CHECK();
                if (j1 < o1) {
                    Opt a; a.overwrite = true; a.btri = true;
                    if (int rc = gemm_on(s4, H + j0 * ld + j1, ld, Ublk + (d + nbk) * OB + (d + nbk), OB, w.tmp, OB, nbk, o1 - j1, o1 - j1, 1.f, a)) return rc;
                    Opt c; c.overwrite = true;
                    if (int rc = gemm_on(s4, dinv_b, NB, w.tmp, OB, Ublk + d * OB + (d + nbk), OB, nbk, o1 - j1, nbk, -1.f, c)) return rc;
                }
            }
            if (j0 > o0) {
                // H[0:j0, o0:j0] -= R[0:j0, b] R[o0:j0, b]^T (columns of this outer block only; tiles below the diagonal
                // skipped).  Right-looking: many short tiles, which keeps this serial chain short.
                Opt uo; uo.nk = true; uo.upper = true; uo.ccol0 = o0;
                if (int rc = gemm_on(s, H + j0, ld, H + o0 * ld + j0, ld, H + o0, ld, j0, j0 - o0, nbk, -1.f, uo)) return rc;
            }
        }
        if (want_inverse && o1 < n) {
            // Still on the stream that trails the chain: R[o, right] <- -U_oo R[o, right], which is what the inverse below
            // needs of this row block.  R[o, right] is final here, no later step of the factorisation reads or writes it,
            // and the product depends on nothing the inverse computes, so it is taken off the inverse's serial path.
            Opt a; a.overwrite = true; a.atri = true;
            if (int rc = gemm_on(s4, Ublk, OB, H + o0 * ld + o1, ld, w.T2, w.ld2, ow, n - o1, ow, -1.f, a)) return rc;
            if (int rc = copy2d(s4, H + o0 * ld + o1, ld, w.T2, w.ld2, ow, n - o1)) return rc;
        }
        // H[0:o0, 0:o0] -= R[0:o0, o] R[0:o0, o]^T (rank 1024, upper tiles), with look-ahead: the columns [p0, o0) of the next
        // outer block are updated first, on the caller's stream, which then goes on to factor that block (short, serial
        // kernels); the rest, H[0:p0, 0:p0], is updated on a helper stream meanwhile.  The two parts and the next block's
        // factorisation write disjoint regions; the next block's own column update waits for the helper's, which wrote
        // the same region.
        if (o0 > 0) {
            const int64_t p0 = o0 - OB;                  // outer blocks start at multiples of OB
            hipEvent_t factored = nullptr;
            if (int rc = ts.mark(s, &factored)) return rc;
            if (int rc = ts.wait(s, rest_done)) return rc;
            rest_done = nullptr;
            // Large updates multiply the bf16 pieces of the panel R[0:o0, o] (gemm_split.hip): one split of the panel serves
            // both parts, as row operand and as column operand.  The plane buffer is free here: its last reader, the
            // previous outer block's rest update, is what the wait above was for.
            const bool split_strip = w.planes && ow == OB && split_pays((o0 / 256) * (OB / 256));
            const bool split_rest = w.planes && ow == OB && p0 > 0 && split_pays((p0 / 256) * (p0 / 256 + 1) / 2);
            if (split_strip || split_rest) {
                if (int rc = launch_split_rows(H + o0, ld, o0, w.planes, s)) return rc;
                if (int rc = ts.mark(s, &factored)) return rc;
            }
            SplitGemm sg{};
            sg.A_planes = sg.B_planes = w.planes;
            sg.A_zero = sg.B_zero = w.planes ? split_zero_block(w.planes, o0) : nullptr;
            sg.ldc = ld; sg.alpha = -1.f;
            if (split_strip) {
                sg.a_panel0 = 0; sg.b_panel0 = (int)(p0 / 256); sg.C = H + p0;
                sg.tiles_m = (int)(o0 / 256); sg.tiles_n = (int)(OB / 256);
                sg.skip_lower = true; sg.crow0 = 0; sg.ccol0 = p0;
                if (int rc = launch_gemm_split(sg, s)) return rc;
            } else {
                Opt co; co.nk = true; co.upper = true; co.ccol0 = p0;
                if (int rc = gemm_on(s, H + o0, ld, H + p0 * ld + o0, ld, H + p0, ld, o0, o0 - p0, ow, -1.f, co)) return rc;
            }
            if (p0 > 0) {
                if (int rc = ts.wait(s2, factored)) return rc;
                if (split_rest) {
                    sg.a_panel0 = sg.b_panel0 = 0; sg.C = H;
                    sg.tiles_m = sg.tiles_n = (int)(p0 / 256);
                    sg.upper_square = true; sg.skip_lower = false;
                    if (int rc = launch_gemm_split(sg, s2)) return rc;
                } else {
                    Opt ro; ro.nk = true; ro.upper = true;
                    if (int rc = gemm_on(s2, H + o0, ld, H + o0, ld, H, ld, p0, p0, ow, -1.f, ro)) return rc;
                }
                if (int rc = ts.mark(s2, &rest_done)) return rc;
            }
        }
    }
    // everything back on the caller's stream
    for (hipStream_t st : {s2, s3, s4}) {
        hipEvent_t done = nullptr;
        if (int rc = ts.mark(st, &done)) return rc;
        if (int rc = ts.wait(s, done)) return rc;
    }

    // Nothing below the diagonal is part of the result (it holds the input's lower half and the below-diagonal parts of
    // straddling update tiles), and the triangular products of the inverse rely on zeros there.
    hipLaunchKernelGGL(zero_lower_kernel, dim3((unsigned)n), dim3(256), 0, s, H, ld, n);
    GPTQ_LAUNCH_CHECK();
    if (!want_inverse) return GPTQ_OK;

    // ---- U = R^-1 in place, right-looking over the outer block columns --------------------------------------------
    hipEvent_t panel_done = nullptr;     // s2: the last column panel, which reuses T
    for (int64_t k = 0; k < nouter; ++k) {
        const int64_t k0 = k * OB, k1 = std::min<int64_t>(k0 + OB, n), kw = k1 - k0;
        const float* Ukk = w.Uoo + k * (int64_t)OB * OB;
        hipEvent_t read_done = nullptr;  // s: the column block above k has been read by this step's update
        bool marked = false;
        if (k1 < n && k0 > 0) {
            // U[0:k0, k1:n] += U[0:k0, k] (-U_kk R[k, k1:n])   (U[0:k0, k] not yet multiplied by U_kk; the second factor is
            // what the factorisation left in the row block)
            if (w.planes && kw == OB && (n - k1) % 256 == 0 && split_pays((k0 / 256) * ((n - k1) / 256))) {
                // through the split products; the column block has been read once its pieces are made
                if (int rc = launch_split_rows(H + k0, ld, k0, w.planes, s)) return rc;
                if (int rc = ts.mark(s, &read_done)) return rc;
                marked = true;
                if (int rc = launch_split_cols(H + k0 * ld + k1, ld, n - k1, w.planes2, s)) return rc;
                SplitGemm sg{};
                sg.A_planes = w.planes; sg.A_zero = split_zero_block(w.planes, k0);
                sg.B_planes = w.planes2; sg.B_zero = split_zero_block(w.planes2, n - k1);
                sg.C = H + k1; sg.ldc = ld; sg.alpha = 1.f; sg.tiles_m = (int)(k0 / 256); sg.tiles_n = (int)((n - k1) / 256);
                if (int rc = launch_gemm_split(sg, s)) return rc;
            } else {
                Opt u;
                if (int rc = gemm_on(s, H + k0, ld, H + k0 * ld + k1, ld, H + k1, ld, k0, n - k1, kw, 1.f, u)) return rc;
            }
        }
        if (!marked) { if (int rc = ts.mark(s, &read_done)) return rc; }
        // On the other stream: U[0:k0, k] <- U[0:k0, k] U_kk through T, and the diagonal block.  Nothing later reads them.
        // The last column block has no update after it: it stays on the caller's stream, with the row-panel buffer (free
        // by now) for its product, beside the last but one on the other stream.
        const bool last = (k == nouter - 1) && nouter > 1;
        hipStream_t sp = last ? s : s2;
        float* Tp = last ? w.T2 : w.T;
        if (!last) { if (int rc = ts.wait(s2, read_done)) return rc; }
        if (k0 > 0) {
            Opt c; c.overwrite = true; c.btri = true;
            if (int rc = gemm_on(sp, H + k0, ld, Ukk, OB, Tp, OB, k0, kw, kw, 1.f, c)) return rc;
            if (int rc = copy2d(sp, H + k0, ld, Tp, OB, k0, kw)) return rc;
        }
        hipLaunchKernelGGL(copy_block_kernel, dim3(256), dim3(256), 0, sp, H + k0 * ld + k0, ld, Ukk, (int64_t)OB, kw, (int)kw, 1);
        GPTQ_LAUNCH_CHECK();
        if (!last) { if (int rc = ts.mark(s2, &panel_done)) return rc; }
    }
    if (int rc = ts.wait(s, panel_done)) return rc;
    return GPTQ_OK;
}

extern "C" int gptq_damp_cholesky_inverse(float* H, int64_t ld, int64_t n, float percdamp,
                                          void* ws, size_t ws_bytes, int* info_dev, void* stream) {
    int rc;
    if (chol_check_args(H, ld, n, percdamp, info_dev, &rc)) return rc;
    if (!ws || !aligned(ws, 256) || ws_bytes < gptq_damp_cholesky_inverse_workspace_bytes(n))
        return fail(GPTQ_ERR_WORKSPACE, "damp_cholesky_inverse: workspace missing, misaligned or too small");
    return chol_run(H, ld, n, percdamp, ws, info_dev, static_cast<hipStream_t>(stream), true);
}

extern "C" size_t gptq_damp_cholesky_workspace_bytes(int64_t n) { return gptq_damp_cholesky_inverse_workspace_bytes(n); }

extern "C" int gptq_damp_cholesky(float* H, int64_t ld, int64_t n, float percdamp,
                                  void* ws, size_t ws_bytes, int* info_dev, void* stream) {
    int rc;
    if (chol_check_args(H, ld, n, percdamp, info_dev, &rc)) return rc;
    if (!ws || !aligned(ws, 256) || ws_bytes < gptq_damp_cholesky_workspace_bytes(n))
        return fail(GPTQ_ERR_WORKSPACE, "damp_cholesky: workspace missing, misaligned or too small");
    return chol_run(H, ld, n, percdamp, ws, info_dev, static_cast<hipStream_t>(stream), true, false);
}

// ---- the variant that allocates nothing -------------------------------------------------------------------
// Same kernels, their workspace in a library-owned device array of fixed size.  Each GPU holds its own copy of the
// array at its own address: the address is looked up once per device, with that device current, and only that
// pointer -- never the array's name, which in host code is a stand-in and no device address -- is handed to kernels.
namespace {
constexpr int64_t NOALLOC_MAX_N = GPTQ_NOALLOC_MAX_N;
constexpr size_t NOALLOC_BYTES = (size_t)(NOALLOC_MAX_N / NB) * NB * NB * sizeof(float)      // inverses of the 128 x 128 diagonal blocks
                                 + 3 * (size_t)NOALLOC_MAX_N * OB * sizeof(float)            // a column panel, a row panel, the U_oo blocks
                                 + (size_t)NB * OB * sizeof(float) + 2048;                   // one row block of a product
static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

constexpr int MAXDEV = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAXDEV] = {};

int scratch_for_current_device(void** out) {
    int dev = 0;
    GPTQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAXDEV) return fail(GPTQ_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        GPTQ_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return fail(GPTQ_ERR_HIP, "hipGetSymbolAddress gave an unusable address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return GPTQ_OK;
}
}  // namespace

extern "C" int64_t gptq_noalloc_max_n(void) { return NOALLOC_MAX_N; }

extern "C" int gptq_damp_cholesky_inverse_noalloc(float* H, int64_t ld, int64_t n, float percdamp, int* info_dev, void* stream) {
    int rc;
    if (chol_check_args(H, ld, n, percdamp, info_dev, &rc)) return rc;
    if (n > NOALLOC_MAX_N)
        return fail(GPTQ_ERR_UNSUPPORTED, "damp_cholesky_inverse_noalloc: n = %lld exceeds the %lld channels the library's static scratch "
                                          "array holds; use gptq_damp_cholesky_inverse with a caller workspace",
                    (long long)n, (long long)NOALLOC_MAX_N);
    static_assert(NOALLOC_MAX_N % OB == 0, "layout below assumes whole outer blocks");
    if (chol_ws_layout(nullptr, n, false).total > NOALLOC_BYTES) return fail(GPTQ_ERR_UNSUPPORTED, "damp_cholesky_inverse_noalloc: scratch layout exceeds the static array");
    void* ws = nullptr;
    if ((rc = scratch_for_current_device(&ws))) return rc;
    return chol_run(H, ld, n, percdamp, ws, info_dev, static_cast<hipStream_t>(stream), false, true, false);
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
