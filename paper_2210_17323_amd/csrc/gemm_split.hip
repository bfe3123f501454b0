// Float32 products of rank 1024 on the bf16 matrix cores: C += alpha * A * B^T with float32 operands, used for the
// deferred rank-1024 updates of the factorisation (Section 3, Step 3: H[rest] -= R[rest, o] R[rest, o]^T) and of
// Alg. 1 (last statement of the outer loop: W[:, later] -= E U[block, later], twice lazily batched).
//
// Every float32 element is the exact sum of three bfloat16 values, a = a1 + a2 + a3 (8 + 8 + 8 significant bits, each
// piece the rounded remainder of the one before), and a product of two such pieces is exact in float32.  Of the nine
// piece products of a * b the six with i + j <= 4 are kept:
//     a b = a1 b1 + (a1 b2 + a2 b1) + (a1 b3 + a2 b2 + a3 b1) + [a2 b3 + a3 b2 + a3 b3, dropped: <= 2^-23 |a b|],
// which is of the size of the rounding a float32 multiply-add commits anyway, and they are accumulated in float32 by
// v_mfma_f32_32x32x16_bf16, smallest first.  The product becomes a bf16 GEMM with K' = 6 K on rearranged operands: at
// 16 times the float32 matrix-core rate per instruction, six times the instructions.
//
// Operands are first split into "planes" (split_rows_kernel for a K-contiguous operand, split_cols_kernel for one
// given as [K x N]) in exactly the blocked layout the Hessian's SYRK kernel consumes: [panel of 256 rows][plane]
// [step of 32 k][256 rows][64 bytes], 16-byte chunks pre-swizzled, so a workgroup's copy of a panel step is 16 linear
// 1 KB transfers straight into LDS.  The kernel is that SYRK kernel's pipeline (256 x 256 tile, 4 wavefronts of
// 128 x 128, five 32 KB LDS stages filled by global_load_lds, one bare barrier per step) with two operand sources, a
// table that says which plane of A meets which plane of B at each of the six passes over K, a rectangular or
// triangular tile grid, and one tile per workgroup (a persistent launch would keep the short serial kernels of the
// other stream off the chip for its whole duration).
#include "common.h"
#include "syrk_tiles.h"

#include <atomic>

namespace gptq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int SK = SPLIT_K;                      // K of a split product
constexpr int PSTEPS = SK / 32;                  // 32-element steps per plane
constexpr int PASSES = 6;
constexpr int REAL_STEPS = PASSES * PSTEPS;      // 192
constexpr int ALL_STEPS = (REAL_STEPS + 4) / 5 * 5;     // 195: whole trips of the five-stage loop; the surplus steps read a block of zeros
constexpr int64_t BLK = 16384;                   // bytes of one (panel, plane, step) block: 256 rows x 64 bytes
constexpr int64_t PANEL_BYTES = 3 * PSTEPS * BLK; // the three planes of one panel of 256 rows
// pass q multiplies plane PLANE_A[q] of A with plane PLANE_B[q] of B (two bits per pass): a3 b1, a1 b3, a2 b2, a2 b1, a1 b2, a1 b1
constexpr unsigned PLANE_A = 2u | (0u << 2) | (1u << 4) | (1u << 6) | (0u << 8) | (0u << 10);
constexpr unsigned PLANE_B = 0u | (2u << 2) | (1u << 4) | (0u << 6) | (1u << 8) | (0u << 10);

__device__ __forceinline__ uint32_t bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// a = p1 + p2 + p3 (each a bfloat16 bit pattern); the two subtractions are exact
__device__ __forceinline__ void split3(float a, uint32_t& p1, uint32_t& p2, uint32_t& p3) {
    p1 = bf16_rne(a);
    float r = a - __uint_as_float(p1 << 16);
    p2 = bf16_rne(r);
    r -= __uint_as_float(p2 << 16);
    p3 = bf16_rne(r);
}

__device__ __forceinline__ unsigned char* plane_block(unsigned char* planes, int64_t panel, int plane, int step) {
    return planes + ((panel * 3 + plane) * PSTEPS + step) * BLK;
}

// A [rows x 1024] float32, K contiguous  ->  planes.  grid (rows / 256, 32 steps); a thread takes 4 consecutive k of one
// row (8 threads a row), so a wavefront reads 8 rows x 128 bytes and writes 8 rows x 64 bytes of each plane.
// Workgroup (0, 0) also clears the block of zeros behind the last panel.
__global__ __launch_bounds__(256) void split_rows_kernel(const float* A, int64_t lda, int64_t rows, unsigned char* planes, int64_t panels) {
    const int64_t panel = blockIdx.x;
    const int step = blockIdx.y;
    if (panel == 0 && step == 0) {
        uint4* z = reinterpret_cast<uint4*>(planes + panels * 3 * PSTEPS * BLK);
#pragma unroll
        for (int i = 0; i < 4; ++i) z[threadIdx.x + 256 * i] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int r = q >> 3, k4 = q & 7;                // row in the panel, which 4 of the step's 32 k
        const int64_t row = panel * 256 + r;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < rows) v = *reinterpret_cast<const float4*>(A + row * lda + step * 32 + k4 * 4);
        uint32_t p[3][4];
        split3(v.x, p[0][0], p[1][0], p[2][0]);
        split3(v.y, p[0][1], p[1][1], p[2][1]);
        split3(v.z, p[0][2], p[1][2], p[2][2]);
        split3(v.w, p[0][3], p[1][3], p[2][3]);
        const int pos = (k4 >> 1) ^ ((r >> 2) & 3);      // swizzled position of this k's 16-byte chunk
        const int off = r * 64 + pos * 16 + (k4 & 1) * 8;
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            *reinterpret_cast<uint2*>(plane_block(planes, panel, pl, step) + off) = make_uint2(p[pl][0] | (p[pl][1] << 16), p[pl][2] | (p[pl][3] << 16));
    }
}

// B [1024 x cols] float32, columns contiguous (a block of rows of an upper-triangular factor)  ->  planes whose "rows"
// are B's columns.  grid (cols / 256, 32 steps): the 32 x 256 piece is read as 1 KB runs, parked in LDS, and every
// thread then owns one column.
__global__ __launch_bounds__(256) void split_cols_kernel(const float* B, int64_t ldb, int64_t cols, unsigned char* planes, int64_t panels) {
    __shared__ float tile[32][256];
    const int64_t panel = blockIdx.x;
    const int step = blockIdx.y;
    if (panel == 0 && step == 0) {
        uint4* z = reinterpret_cast<uint4*>(planes + panels * 3 * PSTEPS * BLK);
#pragma unroll
        for (int i = 0; i < 4; ++i) z[threadIdx.x + 256 * i] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int k = q >> 6, c4 = (q & 63) * 4;
        const int64_t col = panel * 256 + c4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col + 4 <= cols) v = *reinterpret_cast<const float4*>(B + (int64_t)(step * 32 + k) * ldb + col);
        *reinterpret_cast<float4*>(&tile[k][c4]) = v;
    }
    __syncthreads();
    const int r = threadIdx.x;
    uint32_t p[3][32];
#pragma unroll
    for (int k = 0; k < 32; ++k) split3(tile[k][r], p[0][k], p[1][k], p[2][k]);
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
        unsigned char* dst = plane_block(planes, panel, pl, step) + r * 64;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int pos = c ^ ((r >> 2) & 3);
            *reinterpret_cast<uint4*>(dst + pos * 16) = make_uint4(p[pl][8 * c] | (p[pl][8 * c + 1] << 16), p[pl][8 * c + 2] | (p[pl][8 * c + 3] << 16),
                                                                    p[pl][8 * c + 4] | (p[pl][8 * c + 5] << 16), p[pl][8 * c + 6] | (p[pl][8 * c + 7] << 16));
        }
    }
}

struct SplitArgs {
    const unsigned char* Ap;    // planes of A, first panel of the launch
    const unsigned char* Bp;    // planes of B, first panel of the launch
    int64_t zero_off_a, zero_off_b;     // where each operand's 16 KB of zeros lie, in bytes from Ap / Bp (below 2^31)
    float* C; int64_t ldc;
    float alpha;
    int tm, tn;                 // tiles of 256 x 256
    int tri;                    // 1: C square, only the tiles of its upper triangle, numbered in the SYRK kernel's strip order
    int64_t skip_row0, skip_col0;   // rectangular launches: a tile that lies entirely below the diagonal of the parent matrix --
    int skip_lower;                 // its first row past its last column there -- is left out
    int64_t total;              // tiles numbered
    int steps;                  // ALL_STEPS
};

constexpr int DK = 32;
constexpr int DSTAGE = 2 * 256 * DK * 2;            // bytes per stage: A panel step + B panel step
constexpr int PANEL = 256 * DK * 2;

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_split_kernel(SplitArgs g) {
    // separate LDS objects, one per stage: an asynchronous copy into one stage then provably does not alias the operand
    // reads from another
    __shared__ __attribute__((aligned(16))) unsigned char stage0[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage1[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage2[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage3[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage4[DSTAGE];

    // Workgroup w runs on XCD w % 8: a patch of 32 consecutive tiles (~4 x 8 tiles of a strip) goes to one XCD, whose
    // 32 CUs then share the patch's panels in that XCD's L2; consecutive patches go to consecutive XCDs.
    const int64_t w = blockIdx.x;
    const int64_t idx = w >> 3, xcd = w & 7;
    const int64_t L = ((idx >> 5) * 8 + xcd) * 32 + (idx & 31);
    if (L >= g.total) return;
    int bi, bj;
    if (g.tri) {
        syrk_tile_of(g.tm, L, bi, bj);
    } else {
        // strips of 8 tile columns, rows walked top to bottom inside a strip
        const int64_t full = (int64_t)g.tm * STRIP;
        const int s = (int)(L / full);
        const int cols = min(STRIP, g.tn - s * STRIP);
        const int64_t l = L - (int64_t)s * full;
        bi = (int)(l / cols);
        bj = s * STRIP + (int)(l % cols);
        if (g.skip_lower && g.skip_row0 + (int64_t)bi * 256 > g.skip_col0 + (int64_t)bj * 256 + 255) return;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    // A panel step is 16 linear 1 KB runs, four per wavefront.  A lane keeps the address of its 16 bytes of the first run
    // of its panels' first block; the step's two source blocks -- which plane of each operand, or the block of zeros
    // behind the operand's last panel -- are 32-bit offsets from there, the same for every lane.
    const unsigned char* laneA = g.Ap + (int64_t)bi * PANEL_BYTES + wave * 4096 + lane * 16;
    const unsigned char* laneB = g.Bp + (int64_t)bj * PANEL_BYTES + wave * 4096 + lane * 16;
    const uint32_t zeroA = (uint32_t)(g.zero_off_a - (int64_t)bi * PANEL_BYTES);
    const uint32_t zeroB = (uint32_t)(g.zero_off_b - (int64_t)bj * PANEL_BYTES);
    auto issue_copies = [&](unsigned char* stage, int step) {
        unsigned char* base = stage + wave * 4 * 1024;
        const uint32_t q2 = (uint32_t)(step >> 5) * 2u, st = (uint32_t)(step & 31);
        const bool real = step < REAL_STEPS;
        const uint32_t offA = real ? (((PLANE_A >> q2) & 3u) * PSTEPS + st) * (uint32_t)BLK : zeroA;
        const uint32_t offB = real ? (((PLANE_B >> q2) & 3u) * PSTEPS + st) * (uint32_t)BLK : zeroB;
        const unsigned char* sa = laneA + offA;
        const unsigned char* sb = laneB + offB;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(sa + i * 1024),
                                             (__attribute__((address_space(3))) void*)(base + i * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(sb + i * 1024),
                                             (__attribute__((address_space(3))) void*)(base + PANEL + i * 1024), 16, 0, 0);
        }
    };

    floatx16 acc[4][4];
    const int rowA = (wm * 128 + l32) * 64, rowB = PANEL + (wn * 128 + l32) * 64;
    const int co0 = (lhi ^ ((l32 >> 2) & 3)) << 4;
    uint4 fa[2][4], fb[2][4];
    auto fetch = [&](const unsigned char* st, int kk) {
        const int co = co0 ^ (kk << 5);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            fa[kk][s] = *reinterpret_cast<const uint4*>(st + rowA + co + s * 2048);
            fb[kk][s] = *reinterpret_cast<const uint4*>(st + rowB + co + s * 2048);
        }
    };
    auto mma = [&](const uint4& a, const uint4& b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    };
    // One 32-element step out of `cur`: the fragments of its first half are already in fa[0] / fb[0]; those of the second
    // half are fetched while the first 16 MFMAs run, the first fragments of the next step (`nxt`) while the second 16
    // run; the step's 8 copies are spread over its MFMAs (with one wavefront per SIMD nothing else can issue while a
    // copy instruction is being accepted).
    auto multiply = [&](const unsigned char* cur, const unsigned char* nxt) {
        fetch(cur, 1);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[s][u] = mma(fa[0][s], fb[0][u], acc[s][u]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (i & 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        }
        fetch(nxt, 0);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[s][u] = mma(fa[1][s], fb[1][u], acc[s][u]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (i & 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        }
    };
    // A bare s_barrier (a __syncthreads() would drain every outstanding copy).  A step's barrier publishes the stage of
    // the FOLLOWING step: vmcnt(16) = only the 2 x 8 copies of the two steps after that may still be in flight.  The
    // loop body is branch-free: past the last step the copies re-read the block of zeros into a stage nobody multiplies.
    auto next_stage = [&](unsigned char* refill, int step_refill, const unsigned char* cur, const unsigned char* nxt) {
        __builtin_amdgcn_s_waitcnt(0x4F70);             // vmcnt(16)
        asm volatile("s_barrier" ::: "memory");
        issue_copies(refill, min(step_refill, g.steps - 1));
        multiply(cur, nxt);
    };
    issue_copies(stage0, 0);
    issue_copies(stage1, 1);
    issue_copies(stage2, 2);
    issue_copies(stage3, 3);
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][u][i] = 0.f;
    __builtin_amdgcn_s_waitcnt(0x4F78);                 // vmcnt(24): step 0 has landed
    asm volatile("s_barrier" ::: "memory");
    fetch(stage0, 0);
    const int ksteps = g.steps;                         // a multiple of 5, given as an argument: with a constant trip count
                                                        // the compiler restructures the loop and spills accumulators
    for (int ks = 0; ks < ksteps; ks += 5) {
        next_stage(stage4, ks + 4, stage0, stage1);
        next_stage(stage0, ks + 5, stage1, stage2);
        next_stage(stage1, ks + 6, stage2, stage3);
        next_stage(stage2, ks + 7, stage3, stage4);
        next_stage(stage3, ks + 8, stage4, stage0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // the surplus copies have landed before the workgroup ends

    // C += alpha * acc through the memory system's float add: nothing comes back, so nothing waits for a round trip,
    // and every element has one owner in the launch, so it is the same float32 add as a load-add-store.
    const float alpha = g.alpha;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float* cb = g.C + ((int64_t)bi * 256 + wm * 128 + s * 32 + 4 * lhi) * g.ldc + (int64_t)bj * 256 + wn * 128 + u * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) unsafeAtomicAdd(cb + (int64_t)(8 * (i >> 2) + (i & 3)) * g.ldc, alpha * acc[s][u][i]);
        }
}

// A launch takes the split kernel from 144 tiles of 256 x 256 on (one tile per workgroup, one workgroup per CU, ~200 us
// per tile): measured on the 12288-, 14336- and 4096-column layers, a plain minimum anywhere from 96 to 192 tiles gives
// the same times within noise, below that the float32 kernel's smaller tiles fill the chip better.
// gptq_set_split_min_tiles replaces the minimum (tests force the split products onto small matrices).
constexpr int SPLIT_MIN_TILES = 144;
static std::atomic<int> g_split_min_tiles{0};
bool split_pays(int64_t tiles) {
    const int forced = g_split_min_tiles.load(std::memory_order_relaxed);
    return tiles >= (forced > 0 ? forced : SPLIT_MIN_TILES);
}

size_t split_planes_bytes(int64_t rows) {
    const int64_t panels = ceil_div(std::max<int64_t>(rows, 1), 256);
    return (size_t)panels * 3 * PSTEPS * BLK + BLK;
}

int launch_split_rows(const float* A, int64_t lda, int64_t rows, unsigned char* planes, hipStream_t s) {
    if (rows <= 0) return GPTQ_OK;
    if (!aligned(A, 16) || lda % 4 || !aligned(planes, 256)) return fail(GPTQ_ERR_INVALID_ARG, "split_rows: operand not 16-byte aligned");
    const int64_t panels = ceil_div(rows, 256);
    hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)panels, PSTEPS), dim3(256), 0, s, A, lda, rows, planes, panels);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

int launch_split_cols(const float* B, int64_t ldb, int64_t cols, unsigned char* planes, hipStream_t s) {
    if (cols <= 0) return GPTQ_OK;
    if (!aligned(B, 16) || ldb % 4 || cols % 4 || !aligned(planes, 256)) return fail(GPTQ_ERR_INVALID_ARG, "split_cols: operand not 16-byte aligned");
    const int64_t panels = ceil_div(cols, 256);
    hipLaunchKernelGGL(split_cols_kernel, dim3((unsigned)panels, PSTEPS), dim3(256), 0, s, B, ldb, cols, planes, panels);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

int launch_gemm_split(const SplitGemm& p, hipStream_t s) {
    if (p.tiles_m <= 0 || p.tiles_n <= 0) return GPTQ_OK;
    if (p.upper_square && p.tiles_m != p.tiles_n) return fail(GPTQ_ERR_INVALID_ARG, "gemm_split: a triangular launch needs a square C");
    if (!p.A_planes || !p.B_planes || !p.A_zero || !p.B_zero || !p.C || p.ldc < (int64_t)p.tiles_n * 256)
        return fail(GPTQ_ERR_INVALID_ARG, "gemm_split: bad operands");
    SplitArgs g{};
    g.Ap = p.A_planes + (int64_t)p.a_panel0 * 3 * PSTEPS * BLK;
    g.Bp = p.B_planes + (int64_t)p.b_panel0 * 3 * PSTEPS * BLK;
    g.zero_off_a = p.A_zero - g.Ap;
    g.zero_off_b = p.B_zero - g.Bp;
    if (g.zero_off_a < 0 || g.zero_off_b < 0 || g.zero_off_a >= (1LL << 31) || g.zero_off_b >= (1LL << 31))
        return fail(GPTQ_ERR_UNSUPPORTED, "gemm_split: operand too large");
    g.C = p.C; g.ldc = p.ldc; g.alpha = p.alpha;
    g.tm = p.tiles_m; g.tn = p.tiles_n;
    g.tri = p.upper_square ? 1 : 0;
    g.skip_lower = p.skip_lower ? 1 : 0; g.skip_row0 = p.crow0; g.skip_col0 = p.ccol0;
    g.steps = ALL_STEPS;
    g.total = p.upper_square ? syrk_total_tiles(p.tiles_m) : (int64_t)p.tiles_m * p.tiles_n;
    const int64_t blocks = ceil_div(g.total, 256) * 256;       // whole patches of 32 tiles for each of the 8 XCDs
    if (blocks > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "gemm_split: too many tiles");
    hipLaunchKernelGGL(gemm_split_kernel, dim3((unsigned)blocks), dim3(256), 0, s, g);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

}  // namespace gptq

using namespace gptq;

extern "C" int gptq_set_split_min_tiles(int tiles) { return g_split_min_tiles.exchange(tiles > 0 ? tiles : 0); }

// ---- the two deferred updates as calls of their own, through the split products ---------------------------------------
static bool split_call_shapes(int64_t rows, int64_t cols, int64_t k) { return k == SPLIT_K && rows % 256 == 0 && cols % 256 == 0; }

extern "C" size_t gptq_trailing_update_split_workspace_bytes(int64_t r, int64_t ncols) {
    if (r < 0 || ncols < 0) return 0;
    return round_up(split_planes_bytes(r), 256) + round_up(split_planes_bytes(ncols), 256) + 256;
}

extern "C" int gptq_trailing_update_split(float* W, int64_t ldw, const float* E, int64_t lde, const float* U, int64_t ldu,
                                          int64_t r, int64_t ncols, int64_t k, void* ws, size_t ws_bytes, void* stream) {
    if (r < 0 || ncols < 0 || k < 0) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update_split: negative size");
    if (!split_call_shapes(r, ncols, k))
        return fail(GPTQ_ERR_UNSUPPORTED, "trailing_update_split: needs k == %d and r, ncols multiples of 256 (use gptq_trailing_update)", SPLIT_K);
    if (r == 0 || ncols == 0) return GPTQ_OK;
    if (!W || !E || !U) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update_split: null pointer");
    if (ldw < ncols || lde < k || ldu < ncols) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update_split: leading dimension smaller than the row length");
    if (!aligned(W, 16) || !aligned(E, 16) || !aligned(U, 16) || ldw % 4 || lde % 4 || ldu % 4)
        return fail(GPTQ_ERR_INVALID_ARG, "trailing_update_split: W, E and U must be 16-byte aligned with leading dimensions that are multiples of 4");
    if (!ws || !aligned(ws, 256) || ws_bytes < gptq_trailing_update_split_workspace_bytes(r, ncols))
        return fail(GPTQ_ERR_WORKSPACE, "trailing_update_split: workspace missing, misaligned or too small");
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char* pa = static_cast<unsigned char*>(ws);
    unsigned char* pb = pa + round_up(split_planes_bytes(r), 256);
    if (int rc = launch_split_rows(E, lde, r, pa, s)) return rc;
    if (int rc = launch_split_cols(U, ldu, ncols, pb, s)) return rc;
    SplitGemm g{};
    g.A_planes = pa; g.A_zero = split_zero_block(pa, r);
    g.B_planes = pb; g.B_zero = split_zero_block(pb, ncols);
    g.C = W; g.ldc = ldw; g.alpha = -1.f; g.tiles_m = (int)(r / 256); g.tiles_n = (int)(ncols / 256);
    return launch_gemm_split(g, s);
}

extern "C" size_t gptq_symmetric_update_split_workspace_bytes(int64_t n) {
    if (n < 0) return 0;
    return round_up(split_planes_bytes(n), 256) + 256;
}

extern "C" int gptq_symmetric_update_split(float* H, int64_t ldh, const float* P, int64_t ldp, int64_t n, int64_t k,
                                           void* ws, size_t ws_bytes, void* stream) {
    if (n < 0 || k < 0) return fail(GPTQ_ERR_INVALID_ARG, "symmetric_update_split: negative size");
    if (!split_call_shapes(n, n, k))
        return fail(GPTQ_ERR_UNSUPPORTED, "symmetric_update_split: needs k == %d and n a multiple of 256", SPLIT_K);
    if (n == 0) return GPTQ_OK;
    if (!H || !P) return fail(GPTQ_ERR_INVALID_ARG, "symmetric_update_split: null pointer");
    if (ldh < n || ldp < k) return fail(GPTQ_ERR_INVALID_ARG, "symmetric_update_split: leading dimension smaller than the row length");
    if (!aligned(H, 16) || !aligned(P, 16) || ldh % 4 || ldp % 4)
        return fail(GPTQ_ERR_INVALID_ARG, "symmetric_update_split: H and P must be 16-byte aligned with leading dimensions that are multiples of 4");
    if (!ws || !aligned(ws, 256) || ws_bytes < gptq_symmetric_update_split_workspace_bytes(n))
        return fail(GPTQ_ERR_WORKSPACE, "symmetric_update_split: workspace missing, misaligned or too small");
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char* pa = static_cast<unsigned char*>(ws);
    if (int rc = launch_split_rows(P, ldp, n, pa, s)) return rc;
    SplitGemm g{};
    g.A_planes = g.B_planes = pa; g.A_zero = g.B_zero = split_zero_block(pa, n);
    g.C = H; g.ldc = ldh; g.alpha = -1.f; g.tiles_m = g.tiles_n = (int)(n / 256); g.upper_square = true;
    return launch_gemm_split(g, s);
}
