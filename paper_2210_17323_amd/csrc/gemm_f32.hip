// float32 matrix-core GEMM for gfx950, C (+)= alpha * A * op(B).
//
// Used by: the float32 Hessian path, the blocked Cholesky / triangular inverse, and the trailing
// update of Alg. 1 (W[:, i+B:] -= E * Hinv[i:i+B, i+B:]).
//
// Tiling: one workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of C and walks K
// in steps of 16.  Each wavefront owns 64 x 64 = 2 x 2 tiles of v_mfma_f32_32x32x2_f32 (16
// accumulator registers each).  A and B tiles are staged through LDS k-major ([k][m] and [k][n],
// row pitch 132 floats) so that the 32 lanes of a half-wavefront read 32 consecutive floats
// (conflict free); the next K step is prefetched into registers while the current one is multiplied.
#include "common.h"

namespace gptq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int TM = 128, TN = 128, TK = 16, PITCH = 132;

struct GemmArgs {
    const float* A; int64_t lda;
    const float* B; int64_t ldb;
    float* C; int64_t ldc;
    int64_t M, N, K;
    float alpha;
    int overwrite, upper_only;
    int64_t crow0, ccol0;
    int a_upper_tri;
    int b_upper_tri;
    int tiles_m, tiles_n;
    int64_t per_xcd, total;
    int64_t slots;      // tile slots of the launch: per_xcd * 8 (the large-tile kernels may run them on fewer workgroups)
    int tri_ratio;      // > 0: exactly the upper tiles of a square C are enumerated; value = tile rows / tile columns
};

constexpr int GROUP_M = 16;     // tile rows walked fastest inside a group, so co-resident workgroups share B panels
constexpr int NXCD = 8;

// Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (w % 8), so a rectangular launch gives
// each XCD a contiguous range of the tile order; the order walks GROUP_M tile rows fastest, then tile columns.
// Triangular launches are dealt round-robin instead, and have to be dealt EVENLY: every XCD works through its
// own share in order, nothing is stolen.
//  * Upper tiles of a square C (tri_ratio > 0): only the valid tiles are enumerated.  Walking the whole square and
//    returning from the lower tiles gives XCD x the tile rows x and x + 8 of every 16 x 16 diagonal block, 24 - 2x
//    valid tiles: XCD 0 ends up with 10 % more tiles than XCD 7 on a 128-tile-row matrix and the launch ends with
//    most of the chip idle (measured: 89 % instead of 97 % of the CU time busy).
//  * A upper triangular (row-dependent K range): the rows of a group are rotated by the column index, so that
//    every XCD gets every row residue and with it the same mix of long and short tiles.
struct TileOrder {
    // tiles of group gi: a head of ratio*(R-1) columns in which column d holds d/ratio + 1 valid rows, then full columns
    __host__ __device__ static int64_t group_tiles(int tiles_m, int tiles_n, int ratio, int gi, int* rows_out) {
        const int R = (tiles_m - gi * GROUP_M) < GROUP_M ? (tiles_m - gi * GROUP_M) : GROUP_M;
        const int64_t ncols = tiles_n - (int64_t)ratio * GROUP_M * gi;
        *rows_out = R;
        return (int64_t)ratio * R * (R - 1) / 2 + (ncols - (int64_t)ratio * (R - 1)) * R;
    }
    __host__ static int64_t triangle_total(int tiles_m, int tiles_n, int ratio) {
        int64_t t = 0;
        int R;
        for (int gi = 0; gi * GROUP_M < tiles_m; ++gi) t += group_tiles(tiles_m, tiles_n, ratio, gi, &R);
        return t;
    }
    // false: nothing to do for this workgroup.  tm, tn: tile sizes.
    __device__ static bool origin(const GemmArgs& g, int64_t w, int tm, int tn, int64_t& m0, int64_t& n0) {
        int64_t tile = (g.upper_only || g.a_upper_tri) ? w : (w % NXCD) * g.per_xcd + (w / NXCD);
        if (tile >= g.total) return false;
        if (g.tri_ratio > 0) {
            int gi = 0, R;
            for (int64_t c = group_tiles(g.tiles_m, g.tiles_n, g.tri_ratio, 0, &R); tile >= c;
                 c = group_tiles(g.tiles_m, g.tiles_n, g.tri_ratio, gi, &R)) { tile -= c; ++gi; }
            const int64_t head = (int64_t)g.tri_ratio * R * (R - 1) / 2;
            int64_t d, q;
            if (tile < head) {
                d = 0;
                for (int64_t c = 1; tile >= c; c = d / g.tri_ratio + 1) { tile -= c; ++d; }
                q = tile;
            } else {
                tile -= head;
                d = (int64_t)g.tri_ratio * (R - 1) + tile / R;
                q = tile % R;
            }
            m0 = ((int64_t)gi * GROUP_M + q) * tm;
            n0 = ((int64_t)g.tri_ratio * GROUP_M * gi + d) * tn;
        } else {
            const int64_t per_group = (int64_t)GROUP_M * g.tiles_n;
            const int64_t grp = tile / per_group, rem = tile % per_group;
            const int rows = min(GROUP_M, g.tiles_m - (int)grp * GROUP_M);
            int r = (int)(rem % rows);
            if (g.a_upper_tri) r = (int)((r + rem / rows) % rows);
            m0 = (grp * GROUP_M + r) * tm;
            n0 = (rem / rows) * tn;
        }
        return !(g.upper_only && g.crow0 + m0 > g.ccol0 + n0 + (tn - 1));
    }
};

__device__ __forceinline__ float4 load4_guard(const float* p, int64_t valid) {
    // valid = number of in-range elements starting at p (<= 0: none)
    if (valid >= 4) return *reinterpret_cast<const float4*>(p);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (valid > 0) v.x = p[0];
    if (valid > 1) v.y = p[1];
    if (valid > 2) v.z = p[2];
    return v;
}

// The body of one tile.  EDGE = false: the tile lies fully inside C and K is a multiple of TK, so every
// load is an unguarded float4 and the epilogue reads its 16 C values per MFMA tile before it writes any.
template <bool B_IS_NK, bool EDGE>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int64_t m0, const int64_t n0,
                                          float (*As)[TK][PITCH], float (*Bs)[TK][PITCH]) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> register staging: 2 float4 of A and 2 float4 of B per thread per K step
    float4 ra[2], rb[2];
    const float* pa[2];
    const float* pb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = tid + 256 * i;
        pa[i] = g.A + (m0 + (q >> 2)) * g.lda + (q & 3) * 4;
        pb[i] = B_IS_NK ? g.B + (n0 + (q >> 2)) * g.ldb + (q & 3) * 4
                        : g.B + (int64_t)(q >> 5) * g.ldb + n0 + (q & 31) * 4;
    }
    auto load_tiles = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int q = tid + 256 * i;
            if (!EDGE) {
                ra[i] = *reinterpret_cast<const float4*>(pa[i] + k0);
                rb[i] = *reinterpret_cast<const float4*>(B_IS_NK ? pb[i] + k0 : pb[i] + k0 * g.ldb);
            } else {
                const int row = q >> 2, kc = (q & 3) * 4;
                ra[i] = (m0 + row < g.M) ? load4_guard(pa[i] + k0, g.K - (k0 + kc)) : make_float4(0.f, 0.f, 0.f, 0.f);
                if (B_IS_NK) {
                    rb[i] = (n0 + row < g.N) ? load4_guard(pb[i] + k0, g.K - (k0 + kc)) : make_float4(0.f, 0.f, 0.f, 0.f);
                } else {
                    const int krow = q >> 5, nc = (q & 31) * 4;
                    rb[i] = (k0 + krow < g.K) ? load4_guard(pb[i] + k0 * g.ldb, g.N - (n0 + nc)) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int q = tid + 256 * i;
            {
                const int row = q >> 2, kc = (q & 3) * 4;
                As[buf][kc + 0][row] = ra[i].x;
                As[buf][kc + 1][row] = ra[i].y;
                As[buf][kc + 2][row] = ra[i].z;
                As[buf][kc + 3][row] = ra[i].w;
            }
            if (B_IS_NK) {
                const int row = q >> 2, kc = (q & 3) * 4;
                Bs[buf][kc + 0][row] = rb[i].x;
                Bs[buf][kc + 1][row] = rb[i].y;
                Bs[buf][kc + 2][row] = rb[i].z;
                Bs[buf][kc + 3][row] = rb[i].w;
            } else {
                const int krow = q >> 5, nc = (q & 31) * 4;
                *reinterpret_cast<float4*>(&Bs[buf][krow][nc]) = rb[i];
            }
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][t][i] = 0.f;

    const int64_t ksteps = (g.K + TK - 1) / TK;
    // A upper triangular (its row r is zero left of column r): the first m0 columns contribute nothing
    const int64_t ks0 = g.a_upper_tri ? (m0 / TK) : 0;
    load_tiles(ks0 * TK);
    store_tiles(ks0 & 1);
    __syncthreads();

    const int l32 = lane & 31, lhi = lane >> 5;
    for (int64_t ks = ks0; ks < ksteps; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < ksteps) load_tiles((ks + 1) * TK);
        // operand fragments of step kk+1 are read from LDS while the MFMAs of step kk run
        float a[2], b[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) a[s] = As[buf][lhi][wm * 64 + s * 32 + l32];
#pragma unroll
        for (int t = 0; t < 2; ++t) b[t] = Bs[buf][lhi][wn * 64 + t * 32 + l32];
#pragma unroll
        for (int kk = 0; kk < TK / 2; ++kk) {
            float an[2], bn[2];
            if (kk + 1 < TK / 2) {
#pragma unroll
                for (int s = 0; s < 2; ++s) an[s] = As[buf][2 * kk + 2 + lhi][wm * 64 + s * 32 + l32];
#pragma unroll
                for (int t = 0; t < 2; ++t) bn[t] = Bs[buf][2 * kk + 2 + lhi][wn * 64 + t * 32 + l32];
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[s][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[t], acc[s][t], 0, 0, 0);
            if (kk + 1 < TK / 2) {
#pragma unroll
                for (int s = 0; s < 2; ++s) { a[s] = an[s]; b[s] = bn[s]; }
            }
        }
        if (ks + 1 < ksteps) {
            store_tiles(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: accumulator element i of a 32x32 tile is row 8*(i/4) + 4*(lane/32) + i%4, column lane%32
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int64_t col = n0 + wn * 64 + t * 32 + l32;
            const int64_t rbase = m0 + wm * 64 + s * 32 + 4 * lhi;
            float* cbase = g.C + rbase * g.ldc + col;
            if (!EDGE) {
                float cv[16];
                if (!g.overwrite) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) cv[i] = cbase[(int64_t)(8 * (i >> 2) + (i & 3)) * g.ldc];
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float v = g.alpha * acc[s][t][i];
                    cbase[(int64_t)(8 * (i >> 2) + (i & 3)) * g.ldc] = g.overwrite ? v : (cv[i] + v);
                }
            } else {
                if (col >= g.N) continue;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int64_t row = rbase + 8 * (i >> 2) + (i & 3);
                    if (row < g.M) {
                        float* c = g.C + row * g.ldc + col;
                        const float v = g.alpha * acc[s][t][i];
                        *c = g.overwrite ? v : (*c + v);
                    }
                }
            }
        }
}

template <bool B_IS_NK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 3))) void gemm_f32_kernel(GemmArgs g) {
    __shared__ float As[2][TK][PITCH];
    __shared__ float Bs[2][TK][PITCH];
    int64_t m0, n0;
    if (!TileOrder::origin(g, blockIdx.x, TM, TN, m0, n0)) return;
    const bool interior = (m0 + TM <= g.M) && (n0 + TN <= g.N) && (g.K % TK == 0);
    if (interior) gemm_tile<B_IS_NK, false>(g, m0, n0, As, Bs);
    else          gemm_tile<B_IS_NK, true>(g, m0, n0, As, Bs);
}

// ---- large-tile variants: 256 x 128 or 256 x 256 tile, operands copied global -> LDS directly, 4 stages ----
// Used when M % 256 == 0, N % 128 == 0 (256 for the wide tile) and K % 64 == 0.  8 wavefronts, each 64 x 64 = 2 x 2 MFMA tiles.
// A stage holds 16 values of K: the A panel as [256 rows][16 floats] and, for B given as [N x K], the B
// panel as [128 rows][16 floats]; rows are 64 bytes = 4 chunks of 16 bytes, and global_load_lds_dwordx4
// lays 16 such rows down per instruction with the chunk index XOR-swizzled by (row / 4) % 4 on the global
// side: the 16 lanes that a ds_read_b128 serves together read one chunk of 16 consecutive rows, and rows
// 4 apart (256 bytes, the same banks) then sit at different chunk positions -- no bank conflicts.  One 16-byte
// read hands a lane four consecutive k of its row; the half-wavefront h uses chunk 2q+h, and the four
// MFMAs of an octet q consume element i = 0..3 of those reads -- the MFMA's k pairing becomes
// (8q+i, 8q+4+i), the same for A and B, which is all a dot product needs.  For B given as [K x N] the
// stage holds [16 k][128 n] linearly and the matching values are read with ds_read_b32.
// While step k is multiplied, step k+1 has landed (its first fragments are read before step k ends), step
// k+2 is in flight and step k+3 is being issued; one bare s_barrier per step.
constexpr int LM = 256, LN = 128, LK = 16;
constexpr int WIDE_MIN_TILES = 512;
constexpr int LA_BYTES = LM * LK * 4;

// WIDE: the tile is 256 x 256 and a wavefront owns 128 x 64 (4 x 2 MFMA tiles): a third fewer copy instructions and
// a quarter fewer LDS reads per flop, and half as many tile prologues and C read-modify-writes per flop.
template <bool B_IS_NK, bool WIDE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_f32_dma_kernel(GemmArgs g) {
    constexpr int TN_ = WIDE ? 256 : LN;                  // tile columns
    constexpr int SM = WIDE ? 4 : 2;                      // 32-row MFMA tiles per wavefront
    constexpr int NB = TN_ / 128;                         // B copies per wavefront per step
    constexpr int CP = 2 + NB;                            // copies per wavefront per step
    constexpr int LB_ = TN_ * LK * 4, LSTAGE_ = LA_BYTES + LB_;
    __shared__ __attribute__((aligned(16))) unsigned char st0[LSTAGE_];
    __shared__ __attribute__((aligned(16))) unsigned char st1[LSTAGE_];
    __shared__ __attribute__((aligned(16))) unsigned char st2[LSTAGE_];
    __shared__ __attribute__((aligned(16))) unsigned char st3[LSTAGE_];

    // The launch may hold fewer workgroups than tiles (a caller that wants CUs left free for other streams): a
    // workgroup then walks the tile slots w, w + gridDim.x, ...; gridDim.x is a multiple of the XCD count, so all of
    // them are slots of its own XCD's share.
    for (int64_t wslot = blockIdx.x; wslot < g.slots; wslot += gridDim.x) {
    int64_t m0, n0;
    if (!TileOrder::origin(g, wslot, LM, TN_, m0, n0)) continue;

    // 8 wavefronts (two per SIMD, so one can issue MFMAs while the other waits on LDS or the barrier);
    // wavefront (wm, wn) owns rows wm*32*SM.., columns wn*64.. of the tile: SM x 2 MFMA tiles.
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = WIDE ? wave >> 2 : wave >> 1, wn = WIDE ? wave & 3 : wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    // copies: A panel = 16 instructions of 16 rows (2 per wavefront); B panel = 8 or 16 instructions (NB per wavefront):
    // for B given as [N x K] 16 rows each, for [K x N] 1 KB of consecutive n (two k rows of 128, or one of 256)
    const int crow = lane >> 2, cchunk = (lane & 3) ^ ((lane >> 4) & 3);
    const float* srcA = g.A + (m0 + wave * 32 + crow) * g.lda + cchunk * 4;              // + i*16 rows, + k0
    const float* srcB = B_IS_NK ? g.B + (n0 + wave * 16 * NB + crow) * g.ldb + cchunk * 4  // + i*16 rows, + k0
                      : WIDE    ? g.B + (int64_t)(wave * 2) * g.ldb + n0 + lane * 4        // + i k-rows, + k0*ldb
                                : g.B + (int64_t)(wave * 2 + lhi) * g.ldb + n0 + l32 * 4;  // + k0*ldb
    auto issue_copies = [&](unsigned char* stage, int64_t k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcA + (int64_t)i * 16 * g.lda + k0),
                                             (__attribute__((address_space(3))) void*)(stage + (wave * 2 + i) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const float* sb = B_IS_NK ? srcB + (int64_t)i * 16 * g.ldb + k0 : srcB + (k0 + i) * g.ldb;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sb,
                                             (__attribute__((address_space(3))) void*)(stage + LA_BYTES + (wave * NB + i) * 1024), 16, 0, 0);
        }
    };

    floatx16 acc[SM][2];
#pragma unroll
    for (int s = 0; s < SM; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][t][i] = 0.f;

    const int rowA = (wm * 32 * SM + l32) * 64;                  // + s * 2048
    const int rowB = LA_BYTES + (wn * 64 + l32) * 64;            // NK: + t * 2048
    const int swz = (l32 >> 2) & 3;
    const int colB = LA_BYTES + (wn * 64 + l32) * 4;             // KN: + t * 128 + krow * TN_ * 4
    // One 16-deep step out of `cur`.  The fragments of its first 8 k are already in registers (fetched at the
    // end of the previous step); those of the second 8 are read from LDS while the first half's MFMAs run, and
    // the first fragments of the next step (`nxt`, whose copies have landed) while the second half's run.
    float4 a[2][SM];
    float bv[2][2][4];
    auto fetch = [&](const unsigned char* st, int q) {
        const int co = ((2 * q + lhi) ^ swz) << 4;
#pragma unroll
        for (int s = 0; s < SM; ++s) a[q][s] = *reinterpret_cast<const float4*>(st + rowA + s * 2048 + co);
        if (B_IS_NK) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const float4 b4 = *reinterpret_cast<const float4*>(st + rowB + t * 2048 + co);
                bv[q][t][0] = b4.x; bv[q][t][1] = b4.y; bv[q][t][2] = b4.z; bv[q][t][3] = b4.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    bv[q][t][i] = *reinterpret_cast<const float*>(st + colB + t * 128 + (8 * q + 4 * lhi + i) * (TN_ * 4));
        }
    };
    auto mfmas = [&](int q) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int s = 0; s < SM; ++s) {
                const float av = i == 0 ? a[q][s].x : (i == 1 ? a[q][s].y : (i == 2 ? a[q][s].z : a[q][s].w));
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[s][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[q][t][i], acc[s][t], 0, 0, 0);
            }
    };
    auto multiply = [&](const unsigned char* cur, const unsigned char* nxt) {
        fetch(cur, 1);
        mfmas(0);
        // the step's copies (issued by the caller just before) are spread over the first half's MFMAs: the
        // first MFMAs need nothing but registers, so they start right after the barrier instead of behind
        // the copy instructions, each of which holds the wavefront for tens of cycles
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, SM, 0);  // SM MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
            if (i < CP) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);   // 1 copy
        }
        fetch(nxt, 0);
        mfmas(1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, SM, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    // CP copies per wavefront per step.  A step's barrier publishes the stage of the FOLLOWING step (the one
    // `multiply` prefetches from at its end): vmcnt(CP) = only the copies of the step after that may be in flight.
    // Past the last step the copies re-read the last panels into a stage nobody multiplies again.
    const int64_t ks0 = g.a_upper_tri ? m0 / LK : 0;             // A upper triangular: nothing left of the tile's rows
    const int64_t kend = g.b_upper_tri ? min(g.K, n0 + (int64_t)TN_) : g.K;      // B upper triangular: nothing below the tile's last column
    auto next_stage = [&](unsigned char* refill, int64_t k_refill, const unsigned char* cur, const unsigned char* nxt) {
        __builtin_amdgcn_s_waitcnt(0x0F70 | CP);                // vmcnt(CP)
        asm volatile("s_barrier" ::: "memory");
        issue_copies(refill, min(k_refill, kend - LK));
        multiply(cur, nxt);
    };
    issue_copies(st0, ks0 * LK);
    issue_copies(st1, (ks0 + 1) * LK);
    issue_copies(st2, (ks0 + 2) * LK);
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * CP));              // vmcnt(2 CP): step 0 has landed
    asm volatile("s_barrier" ::: "memory");
    fetch(st0, 0);
    for (int64_t k = ks0 * LK; k < kend; k += 4 * LK) {
        next_stage(st3, k + 3 * LK, st0, st1);
        next_stage(st0, k + 4 * LK, st1, st2);
        next_stage(st1, k + 5 * LK, st2, st3);
        next_stage(st2, k + 6 * LK, st3, st0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                         // drain the surplus copies before LDS is released

#pragma unroll
    for (int s = 0; s < SM; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float* cbase = g.C + (m0 + wm * 32 * SM + s * 32 + 4 * lhi) * g.ldc + n0 + wn * 64 + t * 32 + l32;
            float cv[16];
            if (!g.overwrite) {
#pragma unroll
                for (int i = 0; i < 16; ++i) cv[i] = cbase[(int64_t)(8 * (i >> 2) + (i & 3)) * g.ldc];
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float v = g.alpha * acc[s][t][i];
                cbase[(int64_t)(8 * (i >> 2) + (i & 3)) * g.ldc] = g.overwrite ? v : (cv[i] + v);
            }
        }
    __syncthreads();        // the next tile's first copies overwrite the stages this tile's wavefronts still read
    }
}

int launch_gemm_f32(const GemmF32& p, hipStream_t s) {
    if (p.M <= 0 || p.N <= 0) return GPTQ_OK;
    if (!aligned(p.A, 16) || !aligned(p.B, 16) || (p.lda % 4) || (p.ldb % 4))
        return fail(GPTQ_ERR_INVALID_ARG, "gemm_f32: operands must be 16-byte aligned with leading dimensions that are multiples of 4");
    if (p.a_upper_tri && p.K < p.M)
        return fail(GPTQ_ERR_INVALID_ARG, "gemm_f32: an upper-triangular A needs K >= M (the K loop of a tile starts at its first row)");
    GemmArgs g;
    g.A = p.A; g.lda = p.lda; g.B = p.B; g.ldb = p.ldb; g.C = p.C; g.ldc = p.ldc;
    g.M = p.M; g.N = p.N; g.K = p.K < 0 ? 0 : p.K; g.alpha = p.alpha;
    g.overwrite = p.overwrite; g.upper_only = p.upper_only; g.crow0 = p.crow0; g.ccol0 = p.ccol0;
    g.a_upper_tri = p.a_upper_tri;
    g.b_upper_tri = p.b_upper_tri && !p.b_is_nk;
    const bool large = (p.M % LM == 0) && (p.N % LN == 0) && (g.K % (4 * LK) == 0) && g.K > 0 && aligned(p.C, 4);
    // 256 x 256 tiles when they still give every CU a couple of tiles (measured: 3-8 % faster on large rectangular
    // and symmetric-update launches; not on the skinny triangular products, whose tiles differ in K length)
    bool wide = large && !p.a_upper_tri && (p.N % 256 == 0) && (p.M / LM) * (p.N / 256) >= WIDE_MIN_TILES;
    if (large && !wide && !p.a_upper_tri && !p.b_upper_tri && !p.upper_only && (p.N % 256 == 0)) {
        // A rectangular launch of a few rounds: a CU holds one workgroup, so a launch takes ceil(tiles / CUs) rounds of
        // one tile each; the wide tile does 12 % more per cycle (87 against 77 % matrix-core busy cycles).  Take the
        // wide tile where that outweighs the emptier last round.
        const int64_t tw_ = (p.M / LM) * (p.N / 256), tn_ = 2 * tw_;
        const double ew = 0.87 * (double)tw_ / (double)(ceil_div(tw_, 256) * 256);
        const double en = 0.77 * (double)tn_ / (double)(ceil_div(tn_, 256) * 256);
        wide = ew > en;
    }
    const int64_t tm = large ? p.M / LM : ceil_div(p.M, TM), tn = wide ? p.N / 256 : (large ? p.N / LN : ceil_div(p.N, TN));
    if (tm * tn > 0x7ffffff0LL) return fail(GPTQ_ERR_UNSUPPORTED, "gemm_f32: too many tiles");
    g.tiles_m = (int)tm; g.tiles_n = (int)tn;
    g.total = tm * tn;
    g.tri_ratio = 0;
    const int64_t th = large ? LM : TM, tw = wide ? 256 : (large ? LN : TN);      // tile height and width
    if (p.upper_only && p.M == p.N && p.crow0 == p.ccol0 && th % tw == 0 && tn >= tm * (th / tw)) {
        g.tri_ratio = (int)(th / tw);
        g.total = TileOrder::triangle_total(g.tiles_m, g.tiles_n, g.tri_ratio);
    }
    g.per_xcd = ceil_div(g.total, NXCD);
    g.slots = g.per_xcd * NXCD;
    int64_t wgs = g.slots;
    if (large && p.max_workgroups >= NXCD && wgs > p.max_workgroups) wgs = p.max_workgroups / NXCD * NXCD;
    dim3 grid((unsigned)wgs);
    if (large) {
        if (wide) {
            if (p.b_is_nk) hipLaunchKernelGGL((gemm_f32_dma_kernel<true, true>), grid, dim3(512), 0, s, g);
            else           hipLaunchKernelGGL((gemm_f32_dma_kernel<false, true>), grid, dim3(512), 0, s, g);
        } else {
            if (p.b_is_nk) hipLaunchKernelGGL((gemm_f32_dma_kernel<true, false>), grid, dim3(512), 0, s, g);
            else           hipLaunchKernelGGL((gemm_f32_dma_kernel<false, false>), grid, dim3(512), 0, s, g);
        }
    } else {
        if (p.b_is_nk) hipLaunchKernelGGL(gemm_f32_kernel<true>, grid, dim3(256), 0, s, g);
        else           hipLaunchKernelGGL(gemm_f32_kernel<false>, grid, dim3(256), 0, s, g);
    }
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

}  // namespace gptq
