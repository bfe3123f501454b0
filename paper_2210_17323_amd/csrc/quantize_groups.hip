// Step 3 driven by the Cholesky factor R of H + lambda I when the grid is taken per group of 32, 64 or 128 columns
// (Section 4, "Additional Tricks"; Alg. 1): the walk of one block on working weights rebuilt from the accumulators,
// and the inverses of the diagonal blocks of R it needs.  A translation unit of its own: the walk is instantiated per
// group size and weight type, nine long straight-line kernels.
#include "quantize_common.h"

namespace gptq {

// ---- the factor form with grids taken inside a block (groups of 32, 64 or 128 columns) ----------------------------
// A group's grid comes from the weights as they stand when its first column is reached, so the block is walked on
// working weights, as in quant_block_kernel.  At the start of a block they are  w + s U_bb  with U_bb = R_bb^-1, the
// inverse of the block's own 128 x 128 diagonal block of R: the corrections delta of the block's waiting columns
// satisfy delta R_bb = s (the relation of the per-row form, written for every column of the block with the block's
// earlier columns left at their working values), and inside the block Alg. 1 runs on U's diagonal block, which is
// that same R_bb^-1 because U = R^-1 is block upper triangular.  The product s U_bb costs nothing per block: the
// deferred updates run on Rt = R with every column block scaled by its U_bb (scale_column_blocks_kernel, once per call),
// so the accumulators hold  sum_i d_i Rt[i][block] = s U_bb  already.  This kernel adds the original weights, walks the
// block like quant_block_kernel on U_bb, and leaves d_j = w_j - q_j (original weight minus grid value) for the deferred
// updates S[:, later] += D Rt[block, later].
template <typename WT>
struct HybridState {
    WeightRegs<WT> worig;               // original weights of the block
    float w[QB];                        // working weights; d_j once column j is done
    float ring[ustream::RING];
    uint32_t packed[4];
    float e2, scale, zf;
    int zero;
    float* edst;
    uint8_t* cdst;
    bool active;
    __device__ __forceinline__ float (&acc())[QB] { return w; }
};

template <typename WT, int... K>
__device__ __forceinline__ void add_original(HybridState<WT>& st, int nbk, std::integer_sequence<int, K...>) {
    ((st.w[K] = (K < nbk) ? st.w[K] + st.worig.template get<K>() : 0.f), ...);
}

template <int G, int J, typename WT>
__device__ __forceinline__ void hybrid_column(HybridState<WT>& st, lds_floats ubs, const HybridArgs& a, int64_t row, float maxq) {
    if constexpr (J % G == 0) {
        float lo = st.w[J], hi = st.w[J], am = fabsf(st.w[J]);
#pragma unroll
        for (int k = 1; k < G; ++k) {
            lo = fminf(lo, st.w[J + k]); hi = fmaxf(hi, st.w[J + k]); am = fmaxf(am, fabsf(st.w[J + k]));
        }
        grid_from_range(a.grid, maxq, lo, hi, am, st.scale, st.zero);
        st.zf = (float)st.zero;
        if (J < a.nbk) {
            const int64_t gi = (a.j0 + J) / G;
            a.scales[row * a.ngroups + gi] = st.scale;
            a.zeros[row * a.ngroups + gi] = st.zero;
        }
    }
    const float x = st.w[J] / st.scale;
    float c = rintf(x) + st.zf;
    c = fminf(fmaxf(c, 0.f), maxq);
    const float q = __fmul_rn(st.scale, c - st.zf);
    constexpr int diag_slot = ustream::start(J) % ustream::RING;
    const float ujj = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, st.ring[diag_slot]),
                                                                            0x150 + J % ustream::CHUNK, 0xf, 0xf, true));   // row_newbcast
    const float rcp = __builtin_amdgcn_rcpf(ujj);
    const float dw = st.w[J] - q;
    const float e0 = dw * rcp;
    const float e = fmaf(fmaf(-e0, ujj, dw), rcp, e0);      // (w - q) / U[J][J], as in quant_block_kernel
    const float d = st.worig.template get<J>() - q;
    const uint32_t ci = (uint32_t)c;
    if constexpr ((J & 3) == 0) st.packed[(J >> 2) & 3] = ci; else st.packed[(J >> 2) & 3] |= ci << (8 * (J & 3));
    st.e2 = fmaf(e, e, st.e2);
    st.w[J] = d;
    if constexpr ((J & 3) == 3)
        *reinterpret_cast<float4*>(st.edst + J - 3) = make_float4(st.w[J - 3], st.w[J - 2], st.w[J - 1], st.w[J]);
    if constexpr ((J & 15) == 15)
        *reinterpret_cast<uint4*>(st.cdst + J - 15) = make_uint4(st.packed[0], st.packed[1], st.packed[2], st.packed[3]);
    update_row<J>(st, ubs, -e, std::make_integer_sequence<int, ustream::chunks(J)>{});
}

template <int G, typename WT, int... J>
__device__ __forceinline__ void hybrid_columns(HybridState<WT>& st, lds_floats ubs, const HybridArgs& a, int64_t row, float maxq,
                                               std::integer_sequence<int, J...>) {
    (hybrid_column<G, J, WT>(st, ubs, a, row, maxq), ...);
}

template <int G, typename WT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void quant_block_hybrid_kernel(HybridArgs a) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = row < a.r;
    const int64_t rr = active ? row : a.r - 1;
    HybridState<WT> st;
    {
        const float* src = a.T + rr * a.ldt;
        const WT* wsrc = static_cast<const WT*>(a.W) + rr * a.ldw + a.j0;
        if (a.nbk == QB) {
#pragma unroll
            for (int k = 0; k < QB; k += 4) {
                const float4 v = *reinterpret_cast<const float4*>(src + k);
                st.w[k] = v.x; st.w[k + 1] = v.y; st.w[k + 2] = v.z; st.w[k + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < QB; ++k) st.w[k] = (k < a.nbk) ? src[k] : 0.f;
        }
        if constexpr (sizeof(WT) == 2) {
            if (a.nbk == QB && (reinterpret_cast<uintptr_t>(wsrc) & 15) == 0) {
#pragma unroll
                for (int k = 0; k < QB / 2; k += 4) {
                    const uint4 v = *reinterpret_cast<const uint4*>(wsrc + 2 * k);
                    st.worig.v[k] = v.x; st.worig.v[k + 1] = v.y; st.worig.v[k + 2] = v.z; st.worig.v[k + 3] = v.w;
                }
            } else {
                const uint16_t* hsrc = reinterpret_cast<const uint16_t*>(wsrc);
#pragma unroll
                for (int k = 0; k < QB / 2; ++k) {
                    const uint32_t lo = (2 * k < a.nbk) ? hsrc[2 * k] : 0u, hi = (2 * k + 1 < a.nbk) ? hsrc[2 * k + 1] : 0u;
                    st.worig.v[k] = lo | (hi << 16);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < QB; ++k) st.worig.v[k] = (k < a.nbk) ? to_f32<WT>(wsrc[k]) : 0.f;
        }
    }
    __shared__ __align__(16) float ubs[QB * QB];
    stage_diag_block<2>(ubs, a.Ub, QB, 0, QB);
    // working weights = original weights + corrections; columns past a short last block are zero in both
    add_original<WT>(st, a.nbk, std::make_integer_sequence<int, QB>{});
    const float maxq = (float)a.maxq;
    st.scale = 1.f; st.zero = 0; st.zf = 0.f;
    st.e2 = 0.f;
    lds_floats ub = (lds_floats)ubs + (threadIdx.x & 15);
    request_first<HybridState<WT>>(st, ub, std::make_integer_sequence<int, ustream::RING>{});
    st.active = active;
    st.edst = a.D + rr * a.ldd;
    const bool direct = a.nbk == QB && ((reinterpret_cast<uintptr_t>(a.codes + rr * a.ldc + a.j0) & 15) == 0);
    st.cdst = direct ? a.codes + rr * a.ldc + a.j0 : a.cstage + rr * QB;
    hybrid_columns<G, WT>(st, ub, a, rr, maxq, std::make_integer_sequence<int, QB>{});
    const float e2 = st.e2;
    if (!active) return;
    if (!direct) {
        const uint8_t* src = a.cstage + row * QB;
        uint8_t* cdst = a.codes + row * a.ldc + a.j0;
        for (int k = 0; k < a.nbk; ++k) cdst[k] = src[k];
    }
    if (a.half_e2) {
        const double prev = a.first_block ? 0.0 : a.half_e2[row];
        a.half_e2[row] = prev + 0.5 * (double)e2;
    }
}

// U_bb = R_bb^-1 for every 128 x 128 diagonal block of R, dense with zeros below the diagonal and the identity outside
// a short last block.  One workgroup of 128 threads per block; thread c solves R_bb x = e_c from the bottom up
// (x[i] = (delta_ic - sum_{i<k<=c} R[i][k] x[k]) / R[i][i]), R_bb and the columns in LDS.
__global__ __launch_bounds__(128) void invert_diag_blocks_kernel(const float* R, int64_t ldr, int64_t n, float* Ub) {
    extern __shared__ __align__(16) float inv_sm[];
    float* rs = inv_sm;
    float* xs = inv_sm + QB * (QB + 1);
    const int64_t j0 = (int64_t)blockIdx.x * QB;
    const int c = threadIdx.x;
    for (int q = threadIdx.x; q < QB * QB; q += 128) {
        const int i = q / QB, k = q % QB;
        const int64_t gi = j0 + i, gk = j0 + k;
        rs[i * (QB + 1) + k] = (gi < n && gk < n) ? (k >= i ? R[gi * ldr + gk] : 0.f) : (i == k ? 1.f : 0.f);
    }
    __syncthreads();
    for (int i = QB - 1; i > c; --i) xs[i * (QB + 1) + c] = 0.f;
    for (int i = c; i >= 0; --i) {
        float sum = (i == c) ? 1.f : 0.f;
        for (int k = i + 1; k <= c; ++k) sum = fmaf(-rs[i * (QB + 1) + k], xs[k * (QB + 1) + c], sum);
        xs[i * (QB + 1) + c] = sum / rs[i * (QB + 1) + i];
    }
    __syncthreads();
    float* dst = Ub + (int64_t)blockIdx.x * QB * QB;
    for (int q = threadIdx.x; q < QB * QB; q += 128) dst[q] = xs[(q / QB) * (QB + 1) + (q % QB)];
}

// Rt[rows above the block, block] = R[those rows, block] U_bb, one workgroup per 128 x 128 tile above the diagonal
// blocks (tile number t of the strict upper triangle of blocks, column block by column block).  Both operands sit in
// LDS; a thread makes 8 x 4 outputs: its 8 values of a column of A are the same for the 32 threads that share its
// rows (broadcast reads), its 4 values of a row of U_bb one 16-byte read.
__global__ __launch_bounds__(512) void scale_column_blocks_kernel(const float* R, int64_t ldr, int64_t n, const float* Ub, float* Rt, int64_t ldt) {
    int jb = 1, ib = (int)blockIdx.x;                    // tile t -> (ib, jb), ib < jb: column block jb has jb tiles
    while (ib >= jb) { ib -= jb; ++jb; }
    extern __shared__ __align__(16) float scale_sm[];
    constexpr int PA = 133, P = 132;          // pitches: the rows a wavefront reads of A at a time fall on different banks
    float* As = scale_sm;                     // [i][k]
    float* Us = scale_sm + QB * PA;           // [k][c]; 128 * 133 floats is a multiple of 16 bytes
    const int64_t i0 = (int64_t)ib * QB, j0 = (int64_t)jb * QB;
    const float* ub = Ub + (int64_t)jb * QB * QB;
    for (int q = threadIdx.x; q < QB * QB; q += 512) {
        const int i = q / QB, k = q % QB;
        const int64_t gk = j0 + k;
        As[i * PA + k] = (gk < n) ? R[(i0 + i) * ldr + gk] : 0.f;       // rows i0 + i < j0 <= n are inside the matrix
        Us[i * P + k] = ub[q];                                         // row i of U_bb, column k
    }
    __syncthreads();
    const int ty = threadIdx.x >> 5, tx = threadIdx.x & 31;            // rows ty*8 .. +7, columns tx*4 .. +3
    float acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
#pragma unroll 4
    for (int k = 0; k < QB; ++k) {
        float av[8];
#pragma unroll
        for (int a = 0; a < 8; ++a) av[a] = As[(ty * 8 + a) * PA + k];
        const float4 b0 = *reinterpret_cast<const float4*>(Us + k * P + tx * 4);
        const float bv[4] = {b0.x, b0.y, b0.z, b0.w};
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
    }
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        float* dst = Rt + (i0 + ty * 8 + a) * ldt + j0 + tx * 4;
        if (j0 + tx * 4 + 4 <= n) {
            *reinterpret_cast<float4*>(dst) = make_float4(acc[a][0], acc[a][1], acc[a][2], acc[a][3]);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (j0 + tx * 4 + b < n) dst[b] = acc[a][b];
        }
    }
}

int launch_quant_block_hybrid(int64_t group, int wdtype, unsigned workgroups, const HybridArgs& h, hipStream_t s) {
#define GPTQ_HYB(G)                                                                                                                \
    switch (wdtype) {                                                                                                              \
        case GPTQ_F16:  hipLaunchKernelGGL((quant_block_hybrid_kernel<G, _Float16>), dim3(workgroups), dim3(256), 0, s, h); break; \
        case GPTQ_BF16: hipLaunchKernelGGL((quant_block_hybrid_kernel<G, __bf16>),  dim3(workgroups), dim3(256), 0, s, h); break;  \
        default:        hipLaunchKernelGGL((quant_block_hybrid_kernel<G, float>),   dim3(workgroups), dim3(256), 0, s, h); break;  \
    }
    if (group == 32) { GPTQ_HYB(32) } else if (group == 64) { GPTQ_HYB(64) } else if (group == 128) { GPTQ_HYB(128) }
    else return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer_from_factor: group size %lld not built", (long long)group);
#undef GPTQ_HYB
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

int launch_invert_diag_blocks(const float* R, int64_t ldr, int64_t n, float* Ub, hipStream_t s) {
    constexpr size_t inv_lds = 2 * QB * (QB + 1) * sizeof(float);
    GPTQ_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(invert_diag_blocks_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)inv_lds));
    hipLaunchKernelGGL(invert_diag_blocks_kernel, dim3((unsigned)ceil_div(n, QB)), dim3(128), inv_lds, s, R, ldr, n, Ub);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

int launch_scale_column_blocks(const float* R, int64_t ldr, int64_t n, const float* Ub, float* Rt, int64_t ldt, hipStream_t s) {
    const int64_t nblk = ceil_div(n, QB);
    if (nblk < 2) return GPTQ_OK;
    if (nblk > 65535) return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer_from_factor: too many column blocks");
    const int64_t tiles = nblk * (nblk - 1) / 2;
    constexpr size_t lds = (QB * 133 + QB * 132) * sizeof(float);
    GPTQ_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(scale_column_blocks_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(scale_column_blocks_kernel, dim3((unsigned)tiles), dim3(512), lds, s, R, ldr, n, Ub, Rt, ldt);
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

}  // namespace gptq
