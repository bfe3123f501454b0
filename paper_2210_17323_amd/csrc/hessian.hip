// Step 1: H += 2 X X^T  (Section 2, the Hessian of the layer-wise objective; Alg. 1 caption).
//
// X is [n x t] with tokens contiguous, so both operands of X X^T are K-contiguous.  Only tiles of
// the upper triangle of H are computed.  fp16 / bf16 inputs go to v_mfma_f32_32x32x16_{f16,bf16}
// (products exact in float32, float32 accumulation); float32 inputs use the float32 GEMM.
//
// Kernel layout (fp16/bf16): a workgroup owns a BT x BT tile of H and walks the token axis in steps
// of 64.  Per step it stages BT x 64 halves of the row panel and of the column panel in LDS (row
// pitch 128 bytes; the 16-byte chunk index is XOR-swizzled with (row / 2) % 8: a 16-byte access is
// served 16 lanes at a time and rows 2 apart share banks, so both the row-wise stores and the
// one-chunk-of-16-consecutive-rows MFMA operand reads are bank-conflict free), with the next step
// prefetched into registers.  Tiles are enumerated in strips of 8 tile columns
// walked top to bottom and each XCD gets a contiguous range of that order, so the 32 workgroups
// resident on one XCD form a ~4 x 8 patch of tiles that shares its row and column panels in L2.
#include "common.h"
#include "syrk_tiles.h"

namespace gptq {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int HK = 64;          // token step (halves)
constexpr int NXCD = 8;

struct SyrkArgs {
    float* H; int64_t ldh;
    const uint16_t* X; int64_t ldx;
    int64_t n, t;
    int nt;                     // tiles per side
    int64_t total;              // enumerated tile slots (including skipped ones in diagonal patches)
    int64_t per_xcd;
    const unsigned char* Xb;    // repacked copy of the chunk (see repack_kernel), or null: copy straight from X
    int64_t nsteps;             // 32-token steps in the repacked chunk
    // Split token range (direct-to-LDS kernel with a workspace, matrices with few tiles): work item q * total + L
    // is tile L over steps [q * spp, (q + 1) * spp); with splits > 1 an item writes its partial tile to P and
    // syrk_reduce_kernel adds the partials of a tile to H in a fixed order.
    int splits;
    int64_t spp;                // steps per split (a multiple of 5)
    int64_t items;              // total * splits
    float* P;                   // [items][256][256] partial tiles, or null
    // Long calls go through the kernel in slices of the token range (launch_syrk_sliced): while the last of its
    // workgroups still multiply, those that have run out of tiles repack the NEXT slice (next_items > 0), so only
    // the first slice's repack is a pass of its own.
    const uint16_t* next_X;     // first token of the next slice
    int64_t next_t, next_nsteps;
    unsigned char* next_Xb;     // the other half of the workspace
    unsigned int* next_counter; // work counter of that repack, zero when the kernel starts
    unsigned int next_items;    // groups of 16 rows x groups of 512 tokens
    unsigned int next_tgroups;
};

template <bool IS_BF16>
__device__ __forceinline__ floatx16 mfma16(uint4 a, uint4 b, floatx16 c) {
    if constexpr (IS_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
    }
}

__device__ __forceinline__ uint4 load8h_guard(const uint16_t* p, int64_t valid) {
    if (valid >= 8) return *reinterpret_cast<const uint4*>(p);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid <= 0) return v;
    uint16_t h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = (i < valid) ? p[i] : (uint16_t)0;
    v.x = h[0] | ((uint32_t)h[1] << 16);
    v.y = h[2] | ((uint32_t)h[3] << 16);
    v.z = h[4] | ((uint32_t)h[5] << 16);
    v.w = h[6] | ((uint32_t)h[7] << 16);
    return v;
}

// BT: tile side; WM x WN wavefronts; each wavefront owns (BT/WM) x (BT/WN) outputs.
template <bool IS_BF16, int BT, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void syrk_f16_kernel(SyrkArgs g) {
    constexpr int NT = 64 * WM * WN;
    constexpr int SM = BT / WM / 32, SN = BT / WN / 32;      // 32x32 MFMA tiles per wavefront
    constexpr int CH = BT * 8 / NT;                          // 16-byte chunks per thread per panel
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // stage layout: [2][A panel BT*128 bytes | B panel BT*128 bytes]
    constexpr int PANEL = BT * 128;

    // ---- which tile: XCD-contiguous strip order
    const int64_t w = blockIdx.x;
    int64_t L = (w % NXCD) * g.per_xcd + (w / NXCD);
    if (L >= g.total) return;
    int bi, bj;
    syrk_tile_of(g.nt, L, bi, bj);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int64_t r0 = (int64_t)bi * BT, c0 = (int64_t)bj * BT;

    uint4 ra[CH], rb[CH];
    auto load_panels = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int q = tid + NT * i;
            const int row = q >> 3, ch = q & 7;
            const int64_t k = k0 + ch * 8;
            const int64_t ga = r0 + row, gb = c0 + row;
            ra[i] = (ga < g.n) ? load8h_guard(g.X + ga * g.ldx + k, g.t - k) : make_uint4(0, 0, 0, 0);
            rb[i] = (gb < g.n) ? load8h_guard(g.X + gb * g.ldx + k, g.t - k) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_panels = [&](int buf) {
        unsigned char* base = smem + buf * 2 * PANEL;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int q = tid + NT * i;
            const int row = q >> 3, ch = q & 7;
            const int off = row * 128 + ((ch ^ ((row >> 1) & 7)) << 4);
            *reinterpret_cast<uint4*>(base + off) = ra[i];
            *reinterpret_cast<uint4*>(base + PANEL + off) = rb[i];
        }
    };

    floatx16 acc[SM][SN];
#pragma unroll
    for (int s = 0; s < SM; ++s)
#pragma unroll
        for (int u = 0; u < SN; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][u][i] = 0.f;

    const int64_t ksteps = (g.t + HK - 1) / HK;
    load_panels(0);
    store_panels(0);
    __syncthreads();

    for (int64_t ks = 0; ks < ksteps; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < ksteps) load_panels((ks + 1) * HK);
        const unsigned char* pa = smem + buf * 2 * PANEL;
        const unsigned char* pb = pa + PANEL;
#pragma unroll
        for (int kk = 0; kk < HK / 16; ++kk) {
            const int ch = kk * 2 + lhi;
            uint4 fa[SM], fb[SN];
#pragma unroll
            for (int s = 0; s < SM; ++s) {
                const int row = wm * (BT / WM) + s * 32 + l32;
                fa[s] = *reinterpret_cast<const uint4*>(pa + row * 128 + ((ch ^ ((row >> 1) & 7)) << 4));
            }
#pragma unroll
            for (int u = 0; u < SN; ++u) {
                const int row = wn * (BT / WN) + u * 32 + l32;
                fb[u] = *reinterpret_cast<const uint4*>(pb + row * 128 + ((ch ^ ((row >> 1) & 7)) << 4));
            }
#pragma unroll
            for (int s = 0; s < SM; ++s)
#pragma unroll
                for (int u = 0; u < SN; ++u) acc[s][u] = mfma16<IS_BF16>(fa[s], fb[u], acc[s][u]);
        }
        if (ks + 1 < ksteps) {
            store_panels(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- H += 2 * acc
#pragma unroll
    for (int s = 0; s < SM; ++s)
#pragma unroll
        for (int u = 0; u < SN; ++u) {
            const int64_t col = c0 + wn * (BT / WN) + u * 32 + l32;
            if (col >= g.n) continue;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = r0 + wm * (BT / WM) + s * 32 + 8 * (i >> 2) + 4 * lhi + (i & 3);
                if (row < g.n) {
                    float* h = g.H + row * g.ldh + col;
                    *h += 2.0f * acc[s][u][i];
                }
            }
        }
}

// ---- repack of one token chunk into the order the SYRK kernel consumes it -----------------------------
// In X a panel step (256 channels x 32 tokens) is 256 pieces of 64 bytes that lie a whole row apart: every
// piece is its own half cache line, its own DRAM page.  The repacked chunk stores each panel step as one
// contiguous 16 KB block, [panel][step][256 rows][64 bytes], with the 16-byte chunks of a row already in
// their swizzled LDS positions, so a workgroup's copy of a panel step is 16 linear 1 KB transfers.
// Channels past n and tokens past t are zeros (the step count is padded to what the kernel's loop needs).
// Cost: one read and one write of the chunk per call, ~1-2 % of the SYRK.
__global__ __launch_bounds__(256) void repack_kernel(const uint16_t* X, int64_t ldx, int64_t n, int64_t t, int64_t nsteps, unsigned char* Xb) {
    // a workgroup takes 16 rows x 512 tokens: it reads 1 KB runs of each row and writes 1 KB runs of 16 blocks
    const int64_t rg = blockIdx.x;                       // row group of 16
    const int64_t tg = blockIdx.y;                       // token group of 512 (16 steps)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int rr = q >> 6, c64 = q & 63;             // row in group, 16-byte chunk in the 1 KB run
        const int64_t row = rg * 16 + rr;
        const int64_t step = tg * 16 + (c64 >> 2);
        if (step >= nsteps) continue;
        uint4 v = make_uint4(0, 0, 0, 0);
        const int64_t tok = step * 32 + (c64 & 3) * 8;
        if (row < n) v = load8h_guard(X + row * ldx + tok, t - tok);     // zeros past the last token
        const int64_t panel = row >> 8;
        const int r = (int)(row & 255);
        const int pos = (c64 & 3) ^ ((r >> 2) & 3);
        *reinterpret_cast<uint4*>(Xb + (panel * nsteps + step) * 16384 + r * 64 + pos * 16) = v;
    }
}

// The same repacked chunk from token-major activations X[t x n] (channels contiguous: the layout a framework's
// layer input has).  A workgroup turns one panel step -- 32 tokens x 256 channels, read as 512-byte runs of
// each token -- around in LDS and writes it as one contiguous 16 KB block.
__global__ __launch_bounds__(256) void repack_token_major_kernel(const uint16_t* X, int64_t ldx, int64_t n, int64_t t, int64_t nsteps,
                                                                 unsigned char* Xb) {
    __shared__ uint16_t tile[256][32 + 2];               // [channel][token], padded against bank conflicts
    const int64_t panel = blockIdx.x, step = blockIdx.y;
    const int64_t ch0 = panel * 256, tok0 = step * 32;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int tk = q >> 5, c8 = (q & 31) * 8;        // token in the step, first of 8 channels
        uint4 v = make_uint4(0, 0, 0, 0);
        if (tok0 + tk < t) v = load8h_guard(X + (tok0 + tk) * ldx + ch0 + c8, n - (ch0 + c8));    // zeros past the last channel
        const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[c8 + e][tk] = (uint16_t)(wds[e >> 1] >> (16 * (e & 1)));
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int r = q >> 2, c = q & 3;                 // channel in the panel, 16-byte chunk (8 tokens) of its row
        uint32_t wds[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) wds[e] = (uint32_t)tile[r][c * 8 + 2 * e] | ((uint32_t)tile[r][c * 8 + 2 * e + 1] << 16);
        const int pos = c ^ ((r >> 2) & 3);
        *reinterpret_cast<uint4*>(Xb + (panel * nsteps + step) * 16384 + r * 64 + pos * 16) = make_uint4(wds[0], wds[1], wds[2], wds[3]);
    }
}

// ---- 256 x 256 tile, 4 wavefronts of 128 x 128, panels copied global -> LDS directly ----------------
// Each wavefront keeps a 4 x 4 grid of 32x32 accumulators (256 registers), which halves the LDS reads
// per MFMA compared with 128 x 64 wavefront tiles.  The two panels of a 32-token step (2 x 16 KB) go
// straight from global memory into LDS with global_load_lds_dwordx4 (no staging registers, no
// ds_write): one such instruction moves 16 rows x 64 bytes and lays the 64 lanes down linearly in LDS,
// so the XOR swizzle of the 16-byte chunks is applied on the global side (lane l fetches chunk
// (l % 4) ^ ((l / 16) % 4) of row l / 4).  Rows are 64 bytes, so 16 consecutive rows -- what 16 lanes of a
// 16-byte LDS read touch together -- fall on all 16 bank quads exactly when rows 4 apart get different chunk
// positions: the swizzle term is (row / 4) % 4.  Five stages (all 160 KB of LDS): while step k is multiplied the
// copies of steps k+1 .. k+4 are in flight, which is what hides the memory latency with one wavefront per SIMD; one
// barrier per step.  Requires t % 160 == 0 (the caller splits off the tail).
constexpr int DK = 32;                                  // tokens per stage
constexpr int DSTAGE = 2 * 256 * DK * 2;                // bytes per stage: A panel + B panel
constexpr int DMA_TOKENS = 5 * DK;                      // tokens per trip of the 5-stage loop

// The same repack by one wavefront: 16 rows x 512 tokens per work item (16 loads in flight per lane, then 16 stores),
// items handed out by an atomic counter.  Every wavefront that calls this leaves when the counter has passed the last
// item; nobody waits for anybody.
__device__ __forceinline__ void repack_tail(const SyrkArgs& g, int lane) {
    if (g.next_items == 0) return;
    for (;;) {
        unsigned int item = 0;
        if (lane == 0) item = atomicAdd(g.next_counter, 1u);
        item = (unsigned int)__builtin_amdgcn_readfirstlane((int)item);
        if (item >= g.next_items) return;
        const int64_t rg = item / g.next_tgroups, tg = item % g.next_tgroups;
        const int64_t step = tg * 16 + (lane >> 2);
        if (step < g.next_nsteps) {                          // else this lane's 32 tokens lie past the padded slice
            const int64_t tok = step * 32 + (lane & 3) * 8;
            uint4 v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = rg * 16 + i;
                v[i] = make_uint4(0, 0, 0, 0);
                if (row < g.n) v[i] = load8h_guard(g.next_X + row * g.ldx + tok, g.next_t - tok);
            }
            // rows rg*16 .. rg*16+15 lie in one panel (16 divides 256)
            unsigned char* base = g.next_Xb + (((rg * 16) >> 8) * g.next_nsteps + step) * 16384;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = (int)((rg * 16 + i) & 255);
                const int pos = (lane & 3) ^ ((r >> 2) & 3);
                *reinterpret_cast<uint4*>(base + r * 64 + pos * 16) = v[i];
            }
        }
    }
}

template <bool IS_BF16, bool BLOCKED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void syrk_f16_dma_kernel(SyrkArgs g) {
    constexpr int BT = 256;
    constexpr int PANEL = BT * DK * 2;                  // 16 KB
    // Separate LDS objects, one per stage: the compiler then knows that an asynchronous copy into one
    // stage cannot alias the operand reads from another and does not make the reads wait for the copy.
    __shared__ __attribute__((aligned(16))) unsigned char stage0[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage1[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage2[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage3[DSTAGE];
    __shared__ __attribute__((aligned(16))) unsigned char stage4[DSTAGE];      // 5 x 32 KB: all 160 KB of LDS

    const int64_t w = blockIdx.x;
    // Workgroup w runs on XCD w % 8.  A patch = 32 consecutive tile slots (~4 x 8 tiles of one strip) goes to
    // one XCD so that its 32 CUs share the patch's panels in that XCD's L2; consecutive patches go to
    // consecutive XCDs, so at any time the 8 XCDs work on neighbouring row groups of the same strip and find
    // each other's column panels in the memory-side cache instead of HBM.
    // The launch is persistent: 32 workgroups per XCD (one per CU: a workgroup takes all of the LDS), each
    // walking slots w / 8, w / 8 + 32, ... of its XCD, so that the first copies of a workgroup's next tile
    // are on their way while it writes the finished tile out.
    const int64_t xcd = w % NXCD, slot_step = gridDim.x / NXCD;
    int64_t slot = w / NXCD;
    auto tile_at = [&](int64_t sl) { return ((sl / 32) * NXCD + xcd) * 32 + (sl % 32); };
    if (tile_at(slot) >= g.items) {
        if (BLOCKED) repack_tail(g, threadIdx.x & 63);
        return;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    // this lane's part of the 4 + 4 copies of a step: row (wave*4 + i)*16 + lane/4 of each panel, chunk
    // (lane%4) ^ ((lane/16)%4).  Rows past n are clamped: they only feed outputs that are never stored.
    const int lrow = lane >> 2, lchunk = (lane & 3) ^ ((lane >> 4) & 3);
    const uint16_t* xcol = g.X + lchunk * 8;
    int64_t r0 = 0, c0 = 0;                              // origin of the tile whose panels are being copied
    const unsigned char* blkA = nullptr;
    const unsigned char* blkB = nullptr;
    float* part = nullptr;                               // where this item's partial tile goes (split token range)
    auto set_tile = [&](int64_t item) {
        const int64_t q = item / g.total, L = item - q * g.total;
        int bi, bj;
        syrk_tile_of(g.nt, L, bi, bj);
        r0 = (int64_t)bi * BT; c0 = (int64_t)bj * BT;
        if (BLOCKED) {
            blkA = g.Xb + ((int64_t)bi * g.nsteps + q * g.spp) * 16384 + wave * 4096 + lane * 16;
            blkB = g.Xb + ((int64_t)bj * g.nsteps + q * g.spp) * 16384 + wave * 4096 + lane * 16;
            part = g.P ? g.P + item * (int64_t)(BT * BT) : nullptr;
        }
    };
    auto issue_copies = [&](unsigned char* stage, int64_t k0) {
        unsigned char* base = stage + wave * 4 * 1024;
        if (BLOCKED) {
            const int64_t off = (k0 / DK) * 16384;     // this step's block inside the panel
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(blkA + off + i * 1024),
                                                 (__attribute__((address_space(3))) void*)(base + i * 1024), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(blkB + off + i * 1024),
                                                 (__attribute__((address_space(3))) void*)(base + PANEL + i * 1024), 16, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (wave * 4 + i) * 16 + lrow;
            const uint16_t* sa = xcol + min(r0 + row, g.n - 1) * g.ldx + k0;
            const uint16_t* sb = xcol + min(c0 + row, g.n - 1) * g.ldx + k0;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sa,
                                             (__attribute__((address_space(3))) void*)(base + i * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sb,
                                             (__attribute__((address_space(3))) void*)(base + PANEL + i * 1024), 16, 0, 0);
        }
    };

    floatx16 acc[4][4];

    // This lane's operand rows are wm*128 + s*32 + lane%32 (A) and wn*128 + u*32 + lane%32 (B): the swizzle
    // term (row / 4) % 4 is (lane / 4) % 4 for all of them, and s / u only add a constant 2048 bytes.
    const int rowA = (wm * 128 + l32) * 64, rowB = PANEL + (wn * 128 + l32) * 64;
    const int co0 = (lhi ^ ((l32 >> 2) & 3)) << 4;      // chunk offset of sub-step 0; sub-step 1 flips bit 5
    // One 32-token step out of `cur`.  The operand fragments of its first 16 tokens are already in fa[0]/fb[0]
    // (fetched at the end of the previous step); those of the second 16 tokens are fetched from LDS while the
    // first 16 MFMAs run, and the first fragments of the NEXT step (`nxt`, whose copies have landed) while
    // the second 16 run -- so no MFMA ever waits for an LDS round trip, not even right after the barrier.
    // The step's 8 copies are spread over its MFMAs as well: with one wavefront per SIMD nothing else can
    // issue while a copy instruction is being accepted (tens of cycles each), so copies issued back to back
    // idle the matrix core, while one copy every four MFMAs hides behind the MFMA in flight.
    uint4 fa[2][4], fb[2][4];
    auto fetch = [&](const unsigned char* st, int kk) {
        const int co = co0 ^ (kk << 5);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            fa[kk][s] = *reinterpret_cast<const uint4*>(st + rowA + co + s * 2048);
            fb[kk][s] = *reinterpret_cast<const uint4*>(st + rowB + co + s * 2048);
        }
    };
    auto multiply = [&](const unsigned char* cur, const unsigned char* nxt) {
        fetch(cur, 1);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[s][u] = mfma16<IS_BF16>(fa[0][s], fb[0][u], acc[s][u]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // 2 MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
            if (i & 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);   // 1 of this step's 8 copies
        }
        fetch(nxt, 0);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[s][u] = mfma16<IS_BF16>(fa[1][s], fb[1][u], acc[s][u]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (i & 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        }
    };
    // A bare s_barrier: __syncthreads() would also drain every outstanding copy (it fences all memory),
    // which is exactly what the multi-stage pipeline must not do.  Visibility of a stage is established by
    // each wavefront waiting for its own copies of that step before it arrives at the barrier.  A step's
    // barrier publishes the stage of the FOLLOWING step (the one `multiply` prefetches from at its end):
    // vmcnt(16) = only the 2 x 8 copies of the two steps after that may still be in flight.
    // The loop body is branch-free: past the last step the copies simply re-read the last 32 tokens into
    // a stage nobody multiplies again, so every wait is the same.
    auto next_stage = [&](unsigned char* refill, int64_t k_refill, const unsigned char* cur, const unsigned char* nxt) {
        __builtin_amdgcn_s_waitcnt(0x4F70);             // vmcnt(16)
        asm volatile("s_barrier" ::: "memory");         // the next step's stage is complete; everybody left `refill`
        issue_copies(refill, min(k_refill, (g.spp - 1) * DK));
        multiply(cur, nxt);
    };
    const int64_t ksteps = g.spp;                       // a multiple of 5 (the caller pads or splits off the tail)
    set_tile(tile_at(slot));
    issue_copies(stage0, 0);
    issue_copies(stage1, DK);
    issue_copies(stage2, 2 * DK);
    issue_copies(stage3, 3 * DK);
    for (;;) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[s][u][i] = 0.f;
        __builtin_amdgcn_s_waitcnt(0x4F78);             // vmcnt(24): step 0 has landed (and, from the second tile
                                                        // on, the previous tile's updates of H have left)
        asm volatile("s_barrier" ::: "memory");
        fetch(stage0, 0);
        for (int64_t ks = 0; ks < ksteps; ks += 5) {
            next_stage(stage4, (ks + 4) * DK, stage0, stage1);
            next_stage(stage0, (ks + 5) * DK, stage1, stage2);
            next_stage(stage1, (ks + 6) * DK, stage2, stage3);
            next_stage(stage2, (ks + 7) * DK, stage3, stage4);
            next_stage(stage3, (ks + 8) * DK, stage4, stage0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);             // this wavefront's surplus copies have landed: its parts of the stages are free

        // The next tile's first four steps start now.  Another wavefront may still be in its last multiply:
        // that one reads stage 4, which is not refilled here, and prefetches fragments from stage 0 that nobody uses.
        const int64_t er0 = r0, ec0 = c0;
        float* const epart = part;
        slot += slot_step;
        const bool more = tile_at(slot) < g.items;
        if (more) {
            set_tile(tile_at(slot));
            issue_copies(stage0, 0);
            issue_copies(stage1, DK);
            issue_copies(stage2, 2 * DK);
            issue_copies(stage3, 3 * DK);
        }

        // ---- H += 2 * acc with the memory system's float add (no value comes back, so nothing waits for a round
        // trip; reading H first cost ~25 us of exposed latency per 760 us tile).  Each element of H belongs to
        // exactly one tile of the launch, so the sum is the same float32 add in the same order as a load-add-store.
        if (BLOCKED && epart) {
            // split token range: the partial tile as it is, whole (rows and columns past n hold zeros)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float* pb = epart + (wm * 128 + s * 32 + 4 * lhi) * BT + wn * 128 + u * 32 + l32;
#pragma unroll
                    for (int i = 0; i < 16; ++i) pb[(8 * (i >> 2) + (i & 3)) * BT] = acc[s][u][i];
                }
            if (!more) break;
            continue;
        }
        const bool inside = (er0 + BT <= g.n) && (ec0 + BT <= g.n);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t col = ec0 + wn * 128 + u * 32 + l32;
                const int64_t rbase = er0 + wm * 128 + s * 32 + 4 * lhi;
                if (inside) {
                    float* hb = g.H + rbase * g.ldh + col;
#pragma unroll
                    for (int i = 0; i < 16; ++i) unsafeAtomicAdd(hb + (int64_t)(8 * (i >> 2) + (i & 3)) * g.ldh, 2.0f * acc[s][u][i]);
                } else {
                    if (col >= g.n) continue;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int64_t row = rbase + 8 * (i >> 2) + (i & 3);
                        if (row < g.n) unsafeAtomicAdd(g.H + row * g.ldh + col, 2.0f * acc[s][u][i]);
                    }
                }
            }
        if (!more) break;
    }
    if (BLOCKED) repack_tail(g, lane);
}

// H tile += 2 * (P[0] + P[1] + ... + P[splits-1]), the partial tiles of one tile in the order of their token
// ranges.  One workgroup per tile and 32-row slab, one thread per column.
__global__ __launch_bounds__(256) void syrk_reduce_kernel(SyrkArgs g) {
    const int64_t L = blockIdx.x;
    int bi, bj;
    syrk_tile_of(g.nt, L, bi, bj);
    const int64_t col = (int64_t)bj * 256 + threadIdx.x;
    for (int r = 0; r < 32; ++r) {
        const int rt = blockIdx.y * 32 + r;
        const int64_t row = (int64_t)bi * 256 + rt;
        float sum = 0.f;
        for (int q = 0; q < g.splits; ++q) sum += g.P[((int64_t)q * g.total + L) * 65536 + rt * 256 + threadIdx.x];
        if (row < g.n && col < g.n) g.H[row * g.ldh + col] += 2.0f * sum;
    }
}

// How a chunk of t tokens of an n-channel layer goes through the direct-to-LDS kernel with a workspace.
// Matrices with fewer than four 256 x 256 tiles per CU leave much of the chip idle at the end of a launch (or
// all along: n = 4096 has 136 tiles for 256 CUs), so their token range is split into up to 8 parts.  The split
// count minimises a simple cost: rounds of 256 workgroups x (steps per part x 0.76 us + a fixed cost per work
// item: ~8 us to start and to add a tile to H, ~30 us when a partial tile is written, read back and reduced).
struct SyrkPlan { int splits; int64_t nsteps; size_t repack_bytes, partial_bytes; };
static SyrkPlan syrk_plan(int64_t n, int64_t t) {
    const int64_t nt = ceil_div(n, 256), tiles = nt * (nt + 1) / 2, steps = ceil_div(t, DK);
    int best = 1;
    if (tiles < 2048) {
        double best_cost = 0.0;
        for (int S = 1; S <= 8; ++S) {
            if (S > 1 && steps < 20 * (int64_t)S) break;             // a part should be at least 20 steps long
            const double rounds = (double)ceil_div(tiles * S, 256);
            const double cost = rounds * ((double)ceil_div(steps, S) * 0.76 + (S > 1 ? 30.0 : 8.0));
            if (S == 1 || cost < best_cost * 0.98) { best_cost = cost; best = S; }
        }
    }
    SyrkPlan p;
    p.splits = best;
    p.nsteps = ceil_div(steps, 5 * (int64_t)best) * 5 * best;         // zero-padded to whole trips of the 5-stage loop per part
    p.repack_bytes = round_up((size_t)nt * 256 * (size_t)p.nsteps * DK * 2, 256);
    p.partial_bytes = best > 1 ? (size_t)best * tiles * 65536 * sizeof(float) : 0;
    return p;
}

static void syrk_schedule(SyrkArgs& g, int BT) {
    g.nt = (int)ceil_div(g.n, BT);
    g.total = syrk_total_tiles(g.nt);
    g.per_xcd = ceil_div(g.total, NXCD);
}

template <bool IS_BF16>
static int launch_syrk_dma(SyrkArgs g, void* ws, hipStream_t s, bool token_major = false) {
    syrk_schedule(g, 256);
    g.Xb = static_cast<const unsigned char*>(ws);
    g.splits = 1; g.P = nullptr;
    if (ws) {
        const SyrkPlan plan = syrk_plan(g.n, g.t);
        g.splits = plan.splits;
        g.nsteps = plan.nsteps;
        g.spp = g.nsteps / g.splits;
        if (plan.partial_bytes) g.P = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + plan.repack_bytes);
    } else {
        g.nsteps = g.t / DK;
        g.spp = g.nsteps;
    }
    g.items = g.total * g.splits;
    g.per_xcd = ceil_div(ceil_div(g.items, 32), NXCD) * 32;      // whole patches of 32 slots per XCD
    if (g.per_xcd * NXCD > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "hessian: too many tiles");
    const int64_t blocks = std::min<int64_t>(g.per_xcd, 32) * NXCD;   // persistent: one workgroup per CU walks its slots
    if (ws) {
        const int64_t rgroups = (int64_t)g.nt * 16, tgroups = ceil_div(g.nsteps, 16);
        if (tgroups > 65535 || g.nsteps > 65535) return fail(GPTQ_ERR_UNSUPPORTED, "hessian: chunk too long for the repack grid (split the call)");
        if (token_major)
            hipLaunchKernelGGL(repack_token_major_kernel, dim3((unsigned)g.nt, (unsigned)g.nsteps), dim3(256), 0, s, g.X, g.ldx, g.n, g.t,
                               g.nsteps, static_cast<unsigned char*>(ws));
        else
            hipLaunchKernelGGL(repack_kernel, dim3((unsigned)rgroups, (unsigned)tgroups), dim3(256), 0, s, g.X, g.ldx, g.n, g.t, g.nsteps,
                               static_cast<unsigned char*>(ws));
        GPTQ_LAUNCH_CHECK();
        g.t = g.nsteps * DK;
        hipLaunchKernelGGL((syrk_f16_dma_kernel<IS_BF16, true>), dim3((unsigned)blocks), dim3(256), 0, s, g);
        if (g.P) {
            GPTQ_LAUNCH_CHECK();
            hipLaunchKernelGGL(syrk_reduce_kernel, dim3((unsigned)g.total, 8), dim3(256), 0, s, g);
        }
    } else {
        hipLaunchKernelGGL((syrk_f16_dma_kernel<IS_BF16, false>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    }
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

// ---- long calls: the token range in slices, the repack of slice i + 1 inside the kernel of slice i ---------------
// A call with more tokens than one slice goes through the direct-to-LDS kernel slice by slice (the workspace holds two
// repacked slices).  Only the first slice is repacked by a kernel of its own; every later one is repacked by the
// workgroups of the preceding slice's kernel as they run out of tiles (repack_tail), which otherwise sit idle until
// the last workgroup of the launch is through -- 8 % of the launch at n = 12288 (1176 tiles on 256 CUs), about what
// the repack costs.  Taken when one slice alone fills the chip without splitting its token range.
constexpr int64_t SLICE_TOKENS = 32768;
constexpr int MAX_SLICES = 64;

static int64_t slice_tokens() {
    // GPTQ_HESSIAN_SLICE_TOKENS: tokens per slice of a long call (a multiple of 32; default 32768).  Setting it also
    // makes every 16-bit call that is longer than a slice take this path, whatever the matrix size.
    // Read at every call (the workspace query and the call itself must see the same value).
    const char* e = getenv("GPTQ_HESSIAN_SLICE_TOKENS");
    const int64_t x = e ? atoll(e) : 0;
    return (x >= 32 && x % 32 == 0) ? x : 0;
}

static bool syrk_sliced(int64_t n, int64_t t) {
    const int64_t forced = slice_tokens();
    const int64_t slice = forced ? forced : SLICE_TOKENS;
    if (t <= slice || ceil_div(t, slice) > MAX_SLICES) return false;
    return forced != 0 || (n > 6144 && syrk_plan(n, slice).splits == 1);
}

static int64_t padded_steps(int64_t tokens) { return ceil_div(ceil_div(tokens, DK), 5) * 5; }

static size_t syrk_sliced_ws_bytes(int64_t n) {
    const int64_t slice = slice_tokens() ? slice_tokens() : SLICE_TOKENS;
    const size_t one = round_up((size_t)ceil_div(n, 256) * 256 * (size_t)padded_steps(slice) * DK * 2, 256);
    return 2 * one + 256;
}

__global__ void zero_counters_kernel(unsigned int* c, int count) {
    if ((int)threadIdx.x < count) c[threadIdx.x] = 0u;
}

template <bool IS_BF16>
static int launch_syrk_sliced(SyrkArgs g, void* ws, hipStream_t s) {
    const int64_t slice = slice_tokens() ? slice_tokens() : SLICE_TOKENS;
    const int64_t nslices = ceil_div(g.t, slice);
    syrk_schedule(g, 256);
    const size_t one = round_up((size_t)g.nt * 256 * (size_t)padded_steps(slice) * DK * 2, 256);
    unsigned char* buf[2] = {static_cast<unsigned char*>(ws), static_cast<unsigned char*>(ws) + one};
    unsigned int* counters = reinterpret_cast<unsigned int*>(static_cast<unsigned char*>(ws) + 2 * one);
    g.splits = 1; g.P = nullptr;
    g.items = g.total;
    g.per_xcd = ceil_div(ceil_div(g.items, 32), NXCD) * 32;
    if (g.per_xcd * NXCD > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "hessian: too many tiles");
    const int64_t blocks = std::min<int64_t>(g.per_xcd, 32) * NXCD;
    const uint16_t* X0 = g.X;
    const int64_t t_all = g.t;
    hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(MAX_SLICES), 0, s, counters, MAX_SLICES);
    GPTQ_LAUNCH_CHECK();
    {
        const int64_t t0 = std::min<int64_t>(slice, t_all), ns0 = padded_steps(t0);
        hipLaunchKernelGGL(repack_kernel, dim3((unsigned)(g.nt * 16), (unsigned)ceil_div(ns0, 16)), dim3(256), 0, s, X0, g.ldx, g.n, t0, ns0, buf[0]);
        GPTQ_LAUNCH_CHECK();
    }
    for (int64_t i = 0; i < nslices; ++i) {
        const int64_t ti = std::min<int64_t>(slice, t_all - i * slice);
        SyrkArgs a = g;
        a.X = X0 + i * slice;
        a.Xb = buf[i & 1];
        a.nsteps = padded_steps(ti);
        a.spp = a.nsteps;
        a.t = a.nsteps * DK;
        a.next_items = 0;
        if (i + 1 < nslices) {
            const int64_t tn = std::min<int64_t>(slice, t_all - (i + 1) * slice);
            a.next_X = X0 + (i + 1) * slice;
            a.next_t = tn;
            a.next_nsteps = padded_steps(tn);
            a.next_Xb = buf[(i + 1) & 1];
            a.next_counter = counters + i;
            a.next_tgroups = (unsigned int)ceil_div(a.next_nsteps, 16);
            a.next_items = (unsigned int)(g.nt * 16) * a.next_tgroups;
        }
        hipLaunchKernelGGL((syrk_f16_dma_kernel<IS_BF16, true>), dim3((unsigned)blocks), dim3(256), 0, s, a);
        GPTQ_LAUNCH_CHECK();
    }
    return GPTQ_OK;
}

template <bool IS_BF16, int BT, int WM, int WN>
static int launch_syrk(SyrkArgs g, hipStream_t s) {
    g.nt = (int)ceil_div(g.n, BT);
    g.total = syrk_total_tiles(g.nt);
    g.per_xcd = ceil_div(g.total, NXCD);
    const int64_t blocks = g.per_xcd * NXCD;
    if (blocks > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "hessian: too many tiles");
    constexpr size_t lds = 2 * 2 * BT * 128;
    auto kern = syrk_f16_kernel<IS_BF16, BT, WM, WN>;
    GPTQ_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * WM * WN), lds, s, g);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

// ---- mirror the upper triangle onto the lower one, 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void symmetrize_kernel(float* H, int64_t ld, int64_t n) {
    __shared__ float tile[32][33];
    const int64_t bi = blockIdx.y, bj = blockIdx.x;      // source tile (bi, bj) with bj >= bi
    if (bj < bi) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8) {
        const int64_t row = bi * 32 + r, col = bj * 32 + tx;
        tile[r][tx] = (row < n && col < n) ? H[row * ld + col] : 0.f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int64_t row = bj * 32 + r, col = bi * 32 + tx;   // destination (row, col) = source (col, row)
        if (row < n && col < n && row > col) H[row * ld + col] = tile[tx][r];
    }
}

}  // namespace gptq

using namespace gptq;

constexpr int64_t SYRK_DMA_MIN_N = 2048;        // below this even a split token range leaves most CUs without a tile

static size_t syrk_ws_bytes(int64_t n, int64_t t, int xdtype) {
    if (xdtype == GPTQ_F32 || n < SYRK_DMA_MIN_N) return 0;
    if (syrk_sliced(n, t)) return syrk_sliced_ws_bytes(n);
    const SyrkPlan p = syrk_plan(n, t);
    if (n <= 6144 && p.splits == 1) return 0;       // too few tokens to split: the 128-tile kernel does better
    return p.repack_bytes + p.partial_bytes;
}

extern "C" size_t gptq_hessian_accumulate_workspace_bytes(int64_t n, int64_t t, int xdtype) {
    if (n <= 0 || t <= 0) return 0;
    return syrk_ws_bytes(n, t, xdtype);
}

extern "C" int64_t gptq_hessian_accumulate_launches(int64_t n, int64_t t, int xdtype) {
    if (n <= 0 || t <= 0) return 0;
    if (xdtype == GPTQ_F32 || n < SYRK_DMA_MIN_N || !syrk_sliced(n, t)) return 1;
    const int64_t slice = slice_tokens() ? slice_tokens() : SLICE_TOKENS;
    return ceil_div(t, slice);
}

extern "C" int gptq_hessian_accumulate(float* H, int64_t ldh, const void* X, int xdtype,
                                       int64_t n, int64_t t, int64_t ldx, void* ws, size_t ws_bytes, void* stream) {
    if (n < 0 || t < 0) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: negative size");
    if (n == 0 || t == 0) return GPTQ_OK;
    if (!H || !X) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: null pointer");
    if (ldh < n || ldx < t) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: leading dimension smaller than the row length");
    if (xdtype != GPTQ_F16 && xdtype != GPTQ_BF16 && xdtype != GPTQ_F32)
        return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: unknown xdtype %d", xdtype);
    if (!aligned(H, 4)) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: H misaligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (xdtype == GPTQ_F32) {
        if (!aligned(X, 16) || ldx % 4) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: float32 X must be 16-byte aligned with ldx %% 4 == 0");
        GemmF32 g{};
        g.A = static_cast<const float*>(X); g.lda = ldx;
        g.B = g.A; g.ldb = ldx;
        g.C = H; g.ldc = ldh;
        g.M = n; g.N = n; g.K = t; g.alpha = 2.0f;
        g.b_is_nk = true; g.overwrite = false; g.upper_only = true; g.crow0 = 0; g.ccol0 = 0;
        return launch_gemm_f32(g, s);
    }
    if (!aligned(X, 16) || ldx % 8) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate: 16-bit X must be 16-byte aligned with ldx %% 8 == 0");
    SyrkArgs g{};
    g.H = H; g.ldh = ldh; g.X = static_cast<const uint16_t*>(X); g.ldx = ldx; g.n = n; g.t = t;
    const bool bf = xdtype == GPTQ_BF16;
    // With a workspace the chunk is first repacked into contiguous, zero-padded panel steps (much better
    // DRAM-page and cache-line locality for the copies) and the direct-to-LDS kernel takes all of it; matrices
    // with few tiles get their token range split (see syrk_plan).
    const size_t need = syrk_ws_bytes(n, t, xdtype);
    if (need && ws && (!aligned(ws, 256) || ws_bytes < need))
        return fail(GPTQ_ERR_WORKSPACE, "hessian_accumulate: workspace misaligned or smaller than the %zu bytes this call needs "
                                        "(pass NULL to read X in place)", need);
    if (need && ws && syrk_sliced(n, t))
        return bf ? launch_syrk_sliced<true>(g, ws, s) : launch_syrk_sliced<false>(g, ws, s);
    if (need && ws)
        return bf ? launch_syrk_dma<true>(g, ws, s) : launch_syrk_dma<false>(g, ws, s);
    if (n <= 6144)                  // 256-wide tiles only fill the chip when there are enough of them
        return bf ? launch_syrk<true, 128, 2, 2>(g, s) : launch_syrk<false, 128, 2, 2>(g, s);
    // Without one the kernel copies straight from X: whole trips of its 5-stage loop (160 tokens) go through
    // it, the tail through the guarded kernel.
    const int64_t t_main = t / DMA_TOKENS * DMA_TOKENS;
    if (t_main > 0) {
        SyrkArgs gm = g;
        gm.t = t_main;
        const int rc = bf ? launch_syrk_dma<true>(gm, nullptr, s) : launch_syrk_dma<false>(gm, nullptr, s);
        if (rc) return rc;
    }
    if (t_main < t) {
        SyrkArgs gt = g;
        gt.X = g.X + t_main;
        gt.t = t - t_main;
        return bf ? launch_syrk<true, 256, 2, 4>(gt, s) : launch_syrk<false, 256, 2, 4>(gt, s);
    }
    return GPTQ_OK;
}

static size_t syrk_token_major_ws_bytes(int64_t n, int64_t t) {
    const SyrkPlan p = syrk_plan(n, t);
    return p.repack_bytes + p.partial_bytes;
}

extern "C" size_t gptq_hessian_accumulate_token_major_workspace_bytes(int64_t n, int64_t t, int xdtype) {
    if (n <= 0 || t <= 0 || xdtype == GPTQ_F32) return 0;
    return syrk_token_major_ws_bytes(n, t);
}

extern "C" int gptq_hessian_accumulate_token_major(float* H, int64_t ldh, const void* X, int xdtype,
                                                   int64_t n, int64_t t, int64_t ldx, void* ws, size_t ws_bytes, void* stream) {
    if (n < 0 || t < 0) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: negative size");
    if (n == 0 || t == 0) return GPTQ_OK;
    if (!H || !X) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: null pointer");
    if (ldh < n || ldx < n) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: leading dimension smaller than the row length");
    if (xdtype == GPTQ_F32) return fail(GPTQ_ERR_UNSUPPORTED, "hessian_accumulate_token_major: float32 activations are only taken channel-major");
    if (xdtype != GPTQ_F16 && xdtype != GPTQ_BF16) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: unknown xdtype %d", xdtype);
    if (!aligned(H, 4)) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: H misaligned");
    if (!aligned(X, 16) || ldx % 8) return fail(GPTQ_ERR_INVALID_ARG, "hessian_accumulate_token_major: X must be 16-byte aligned with ldx %% 8 == 0");
    if (!ws || !aligned(ws, 256) || ws_bytes < syrk_token_major_ws_bytes(n, t))
        return fail(GPTQ_ERR_WORKSPACE, "hessian_accumulate_token_major: workspace missing, misaligned or too small");
    SyrkArgs g{};
    g.H = H; g.ldh = ldh; g.X = static_cast<const uint16_t*>(X); g.ldx = ldx; g.n = n; g.t = t;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return xdtype == GPTQ_BF16 ? launch_syrk_dma<true>(g, ws, s, true) : launch_syrk_dma<false>(g, ws, s, true);
}

extern "C" int gptq_hessian_symmetrize(float* H, int64_t ldh, int64_t n, void* stream) {
    if (n < 0) return fail(GPTQ_ERR_INVALID_ARG, "hessian_symmetrize: negative size");
    if (n == 0) return GPTQ_OK;
    if (!H || ldh < n) return fail(GPTQ_ERR_INVALID_ARG, "hessian_symmetrize: bad H / ldh");
    const int64_t nb = ceil_div(n, 32);
    if (nb > 65535) return fail(GPTQ_ERR_UNSUPPORTED, "hessian_symmetrize: n too large");
    hipLaunchKernelGGL(symmetrize_kernel, dim3((unsigned)nb, (unsigned)nb), dim3(256), 0, static_cast<hipStream_t>(stream), H, ldh, n);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}
