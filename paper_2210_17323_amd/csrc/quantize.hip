// Step 3: Algorithm 1 -- column-by-column quantization in lazy blocks of B = 128 with error
// propagation (Section 3, Steps 1-3; Alg. 1), grids of Section 4 (Setup; grouping; "Extreme
// Quantization").
//
// Per block of 128 columns:
//   quant_block_kernel : one LANE per weight row.  The lane keeps its 128 working weights in
//       registers and walks the columns in order: code = clamp(rint(w/scale) + zero), q = grid
//       value, e = (w - q) / U[j][j], then w[k] -= e * U[j][k] for the later columns of the block.
//       Rows are independent (the Hessian information U is shared by all rows), so there is no
//       cross-lane traffic between rows; the 128 x 128 block of U is the same for every lane: the
//       workgroup copies it into LDS once, 16 consecutive values of a row of U are read into one
//       register spread over 16 lanes, and each multiply-add picks its value out of that register with
//       the DPP row broadcast.  The column loop is unrolled by template recursion so every register
//       index is static.  Outputs: codes, the block's error matrix E (r x 128), per-row sum of e^2.
//   trailing update    : W[:, i+B:] -= E * U[i:i+B, i+B:], the float32 matrix-core GEMM, applied at once to
//       the rest of the current 1024-column outer block and deferred (rank 1024) for the columns beyond.
#include "quantize_common.h"

namespace gptq {

// One workgroup per row: convert the row and reduce min / max / max|.|.
template <typename T>
__global__ __launch_bounds__(256) void prepare_rows_kernel(const T* W, int64_t ldw, int64_t n, float* Wk, int64_t ldk,
                                                           int want_grid, int grid, float maxq, float* scales, int32_t* zeros) {
    const int64_t row = blockIdx.x;
    float lo = INFINITY, hi = -INFINITY, am = 0.f;
    for (int64_t k = threadIdx.x; k < n; k += 256) {
        const float v = to_f32<T>(W[row * ldw + k]);
        Wk[row * ldk + k] = v;
        lo = fminf(lo, v); hi = fmaxf(hi, v); am = fmaxf(am, fabsf(v));
    }
    if (!want_grid) return;
    __shared__ float slo[256], shi[256], sam[256];
    slo[threadIdx.x] = lo; shi[threadIdx.x] = hi; sam[threadIdx.x] = am;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            slo[threadIdx.x] = fminf(slo[threadIdx.x], slo[threadIdx.x + w]);
            shi[threadIdx.x] = fmaxf(shi[threadIdx.x], shi[threadIdx.x + w]);
            sam[threadIdx.x] = fmaxf(sam[threadIdx.x], sam[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float sc; int zr;
        grid_from_range(grid, maxq, slo[0], shi[0], sam[0], sc, zr);
        scales[row] = sc; zeros[row] = zr;
    }
}

// Grid of one group that spans several blocks (group % 128 == 0): one wavefront per row over the
// current working weights W[:, j : j+g].
__global__ __launch_bounds__(64) void group_grid_kernel(const float* Wk, int64_t ldk, int64_t j, int64_t g, int grid, float maxq,
                                                        float* scales, int32_t* zeros, int64_t ngroups, int64_t gidx) {
    const int64_t row = blockIdx.x;
    float lo = INFINITY, hi = -INFINITY, am = 0.f;
    for (int64_t k = threadIdx.x; k < g; k += 64) {
        const float v = Wk[row * ldk + j + k];
        lo = fminf(lo, v); hi = fmaxf(hi, v); am = fmaxf(am, fabsf(v));
    }
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
        am = fmaxf(am, __shfl_xor(am, off));
    }
    if (threadIdx.x == 0) {
        float sc; int zr;
        grid_from_range(grid, maxq, lo, hi, am, sc, zr);
        scales[row * ngroups + gidx] = sc; zeros[row * ngroups + gidx] = zr;
    }
}

struct QuantArgs {
    float* Wk; int64_t ldk;         // working weights, points at column 0
    const float* U; int64_t ldu;    // the factor, points at U[0][0]
    int64_t r, n, j0; int nbk;
    int grid; int maxq;
    float* scales; int32_t* zeros; int64_t ngroups;   // [r x ngroups]
    int64_t group;                  // 0 or the group size
    uint8_t* codes; int64_t ldc;
    float* E; int64_t lde;          // this block's 128 columns of the outer error matrix [r x 1024]
    double* half_e2;                // [r] or null
    int first_block;
};

struct QuantState {
    float w[QB];                        // working weights of the block; e_j once column j is done
    float ring[ustream::RING];
    uint32_t packed[QB / 4];            // codes, four to a word
    float e2, scale, zf;
    int zero;
    float* edst;                        // this row of the block's error matrix
    bool active;                        // row inside the matrix
    __device__ __forceinline__ float (&acc())[QB] { return w; }      // what the rank-1 updates of a column go to
};

// The same walk driven by the Cholesky factor R of H + lambda I itself instead of U = R^-1 (see quant_block_rf_kernel):
// the original weights stay as they are and the updates go to an accumulator s[k] = sum over quantized i of d_i R[i][k].
template <typename WT>
struct FactorState {
    WeightRegs<WT> w;                   // original weights of the block
    float s[QB];                        // accumulators; d_j = w_j - q_j once column j is done
    float ring[ustream::RING];
    uint32_t packed[4];                 // codes of the current 16 columns, four to a word
    float e2, scale, zf;
    int zero;
    float* edst;                        // this row of the block's matrix of d
    uint8_t* cdst;                      // this row's codes of the block (16-byte aligned) or null
    bool active;
    __device__ __forceinline__ float (&acc())[QB] { return s; }
};

// Column J of the block: its grid if a group starts here, the code, the error, the update of the columns right of it.
template <int G, int J>
__device__ __forceinline__ void quantize_column(QuantState& st, lds_floats ubs, const QuantArgs& a, int64_t row, float maxq) {
    if constexpr (G > 0 && J % (G > 0 ? G : 1) == 0) {
        float lo = st.w[J], hi = st.w[J], am = fabsf(st.w[J]);
#pragma unroll
        for (int k = 1; k < G; ++k) {
            lo = fminf(lo, st.w[J + k]); hi = fmaxf(hi, st.w[J + k]); am = fmaxf(am, fabsf(st.w[J + k]));
        }
        grid_from_range(a.grid, maxq, lo, hi, am, st.scale, st.zero);
        st.zf = (float)st.zero;
        if (J < a.nbk) {                                    // same for all lanes; lanes past the last row: see the stores of E
            const int64_t gi = (a.j0 + J) / (G > 0 ? G : 1);
            a.scales[row * a.ngroups + gi] = st.scale;
            a.zeros[row * a.ngroups + gi] = st.zero;
        }
    }
    const float x = st.w[J] / st.scale;
    float c = rintf(x) + st.zf;
    c = fminf(fmaxf(c, 0.f), maxq);
    const float q = __fmul_rn(st.scale, c - st.zf);        // the grid value, rounded on its own (never fused into w - q)
    // e = (w - q) / U[J][J]: reciprocal estimate, then one correction step with the exact remainder -- the
    // rounded quotient at a third of the instructions of the general division (no range scaling: U[J][J] is
    // the square root of a diagonal element of the inverse Hessian, far from the ends of the float range)
    constexpr int diag_slot = ustream::start(J) % ustream::RING;        // row J's first chunk holds U[J][J]
    const float ujj = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, st.ring[diag_slot]),
                                                                            0x150 + J % ustream::CHUNK, 0xf, 0xf, true));   // row_newbcast
    const float rcp = __builtin_amdgcn_rcpf(ujj);
    const float d = st.w[J] - q;
    const float e0 = d * rcp;
    const float e = fmaf(fmaf(-e0, ujj, d), rcp, e0);
    const uint32_t ci = (uint32_t)c;
    if constexpr ((J & 3) == 0) st.packed[J >> 2] = ci; else st.packed[J >> 2] |= ci << (8 * (J & 3));
    st.e2 = fmaf(e, e, st.e2);
    st.w[J] = e;
    // Finished columns of E leave four at a time, which frees their registers.  No test of `active` here (it
    // would cut the straight line into pieces): lanes past the last row work on a copy of the last row and
    // store the same values to the same place as that row's own lane.
    if constexpr ((J & 3) == 3)
        *reinterpret_cast<float4*>(st.edst + J - 3) = make_float4(st.w[J - 3], st.w[J - 2], st.w[J - 1], st.w[J]);
    update_row<J>(st, ubs, -e, std::make_integer_sequence<int, ustream::chunks(J)>{});
}

template <int G, int... J>
__device__ __forceinline__ void quantize_columns(QuantState& st, lds_floats ubs, const QuantArgs& a, int64_t row, float maxq,
                                                 std::integer_sequence<int, J...>) {
    (quantize_column<G, J>(st, ubs, a, row, maxq), ...);
}

// G = 0: the grid of this block's columns is already in scales/zeros (per-row grid, or a group of
//        several blocks).  G in {8,16,32,64,128}: groups inside the block, grid taken from the
//        current register values at each group start.
template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void quant_block_kernel(QuantArgs a) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = row < a.r;
    const int64_t rr = active ? row : a.r - 1;
    // This lane's 128 working weights first: 32 scattered 16-byte loads (lanes are a whole row apart) whose round
    // trips then overlap the staging of U below.
    QuantState st;
    float (&w)[QB] = st.w;
    {
        const float* src = a.Wk + rr * a.ldk + a.j0;
        if (a.nbk == QB) {
#pragma unroll
            for (int k = 0; k < QB; k += 4) {
                const float4 v = *reinterpret_cast<const float4*>(src + k);
                w[k] = v.x; w[k + 1] = v.y; w[k + 2] = v.z; w[k + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < QB; ++k) w[k] = (k < a.nbk) ? src[k] : 0.f;
        }
    }
    __shared__ __align__(16) float ubs[QB * QB];
    stage_diag_block<1>(ubs, a.U, a.ldu, a.j0, a.n);
    const float maxq = (float)a.maxq;
    st.scale = 1.f; st.zero = 0;
    if (G == 0) {
        const int64_t gi = a.group ? (a.j0 / a.group) : 0;
        st.scale = a.scales[rr * a.ngroups + gi];
        st.zero = a.zeros[rr * a.ngroups + gi];
    }
    st.zf = (float)st.zero;
    st.e2 = 0.f;
    lds_floats ub = (lds_floats)ubs + (threadIdx.x & 15);           // this lane's element of every chunk
    request_first<QuantState>(st, ub, std::make_integer_sequence<int, ustream::RING>{});
    st.active = active;
    st.edst = a.E + rr * a.lde;
    quantize_columns<G>(st, ub, a, rr, maxq, std::make_integer_sequence<int, QB>{});
    const float e2 = st.e2;
    if (!active) return;
    uint32_t (&packed)[QB / 4] = st.packed;
    uint8_t* cdst = a.codes + row * a.ldc + a.j0;
    if (a.nbk == QB && (reinterpret_cast<uintptr_t>(cdst) & 15) == 0) {
#pragma unroll
        for (int k = 0; k < QB / 4; k += 4)
            *reinterpret_cast<uint4*>(cdst + 4 * k) = make_uint4(packed[k], packed[k + 1], packed[k + 2], packed[k + 3]);
    } else {
#pragma unroll
        for (int k = 0; k < QB; ++k)
            if (k < a.nbk) cdst[k] = (uint8_t)((packed[k >> 2] >> (8 * (k & 3))) & 0xff);
    }
    if (a.half_e2) {
        const double prev = a.first_block ? 0.0 : a.half_e2[row];
        a.half_e2[row] = prev + 0.5 * (double)e2;
    }
}

// ---- the factor form: Alg. 1 driven by R, the Cholesky factor of H + lambda I itself (H + lambda I = R R^T) -------
// U = R^-1 is never formed.  With d_i = w_i - q_i (original weight minus grid value) for the columns already
// quantized, the weight Alg. 1 holds at column j is  w_j + s_j / R[j][j],  s_j = sum_{i<j} d_i R[i][j]  -- the
// unique correction that keeps (delta R)_k = 0 for the columns still free -- and Alg. 1's scaled error is
// e_j = (that weight - q_j) R[j][j], since U[j][j] = 1 / R[j][j].  So the walk is the same as above with other
// operands: the original weights stay untouched in registers, the rank-1 update of a column adds d_j R[j][k] to the
// accumulators s[k], and the deferred updates are S[:, later] += D R[block, later] on the matrix cores.
// One grid per row only (it comes from the original weights): a grid taken from the current weights in the middle of
// the walk would need the waiting columns' corrections, a triangular solve per group start.
struct FactorArgs {
    const void* W; int64_t ldw;     // original weights, type WT
    float* S; int64_t lds_;         // accumulators [r x n] (leading dimension lds_)
    const float* R; int64_t ldr;
    int64_t r, n, j0; int nbk;
    int maxq;
    const float* scales; const int32_t* zeros;      // [r]
    uint8_t* codes; int64_t ldc;
    uint8_t* cstage;                // [r x 128] bytes, 16-byte aligned: codes of a block that cannot be stored in place 16 at a time
    float* D; int64_t ldd;          // this block's 128 columns of the outer matrix of d [r x 1024]
    double* half_e2;
    int first_block;
};

template <int J, typename WT>
__device__ __forceinline__ void factor_column(FactorState<WT>& st, lds_floats ubs, float maxq) {
    constexpr int diag_slot = ustream::start(J) % ustream::RING;        // row J's first chunk holds R[J][J]
    const float rjj = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, st.ring[diag_slot]),
                                                                            0x150 + J % ustream::CHUNK, 0xf, 0xf, true));   // row_newbcast
    // s_j / R[J][J]: reciprocal estimate and one correction step with the exact remainder (the rounded quotient
    // without the range scaling of a general division; R[J][J] is the square root of a pivot of the damped Hessian)
    const float rcp = __builtin_amdgcn_rcpf(rjj);
    const float sj = st.s[J];
    const float t0 = sj * rcp;
    const float wj = st.w.template get<J>();
    const float wn = wj + fmaf(fmaf(-t0, rjj, sj), rcp, t0);           // the weight Alg. 1 holds at this column
    const float x = wn / st.scale;
    float c = rintf(x) + st.zf;
    c = fminf(fmaxf(c, 0.f), maxq);
    const float q = __fmul_rn(st.scale, c - st.zf);
    const float d = wj - q;
    const float e = (wn - q) * rjj;
    const uint32_t ci = (uint32_t)c;
    if constexpr ((J & 3) == 0) st.packed[(J >> 2) & 3] = ci; else st.packed[(J >> 2) & 3] |= ci << (8 * (J & 3));
    st.e2 = fmaf(e, e, st.e2);
    st.s[J] = d;
    // Finished columns leave as they go, which frees their registers: d four at a time, codes sixteen at a time.  No
    // test of `active` (it would cut the straight line into pieces): lanes past the last row work on a copy of the
    // last row and store the same values to the same place as that row's own lane.
    if constexpr ((J & 3) == 3)
        *reinterpret_cast<float4*>(st.edst + J - 3) = make_float4(st.s[J - 3], st.s[J - 2], st.s[J - 1], st.s[J]);
    if constexpr ((J & 15) == 15)
        *reinterpret_cast<uint4*>(st.cdst + J - 15) = make_uint4(st.packed[0], st.packed[1], st.packed[2], st.packed[3]);
    update_row<J>(st, ubs, d, std::make_integer_sequence<int, ustream::chunks(J)>{});
}

template <typename WT, int... J>
__device__ __forceinline__ void factor_columns(FactorState<WT>& st, lds_floats ubs, float maxq, std::integer_sequence<int, J...>) {
    (factor_column<J>(st, ubs, maxq), ...);
}

template <typename WT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void quant_block_rf_kernel(FactorArgs a) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = row < a.r;
    const int64_t rr = active ? row : a.r - 1;
    FactorState<WT> st;
    {
        // This lane's accumulators and original weights first (scattered loads, lanes are a whole row apart): their
        // round trips overlap the staging of R below, which goes in two passes to stay inside the register file.
        const float* src = a.S + rr * a.lds_ + a.j0;
        const WT* wsrc = static_cast<const WT*>(a.W) + rr * a.ldw + a.j0;
        if (a.nbk == QB) {
#pragma unroll
            for (int k = 0; k < QB; k += 4) {
                const float4 v = *reinterpret_cast<const float4*>(src + k);
                st.s[k] = v.x; st.s[k + 1] = v.y; st.s[k + 2] = v.z; st.s[k + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < QB; ++k) st.s[k] = (k < a.nbk) ? src[k] : 0.f;
        }
        if constexpr (sizeof(WT) == 2) {
            if (a.nbk == QB && (reinterpret_cast<uintptr_t>(wsrc) & 15) == 0) {
#pragma unroll
                for (int k = 0; k < QB / 2; k += 4) {
                    const uint4 v = *reinterpret_cast<const uint4*>(wsrc + 2 * k);
                    st.w.v[k] = v.x; st.w.v[k + 1] = v.y; st.w.v[k + 2] = v.z; st.w.v[k + 3] = v.w;
                }
            } else {
                const uint16_t* hsrc = reinterpret_cast<const uint16_t*>(wsrc);
#pragma unroll
                for (int k = 0; k < QB / 2; ++k) {
                    const uint32_t lo = (2 * k < a.nbk) ? hsrc[2 * k] : 0u, hi = (2 * k + 1 < a.nbk) ? hsrc[2 * k + 1] : 0u;
                    st.w.v[k] = lo | (hi << 16);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < QB; ++k) st.w.v[k] = (k < a.nbk) ? to_f32<WT>(wsrc[k]) : 0.f;
        }
    }
    __shared__ __align__(16) float ubs[QB * QB];
    stage_diag_block<2>(ubs, a.R, a.ldr, a.j0, a.n);
    const float maxq = (float)a.maxq;
    st.scale = a.scales[rr];
    st.zero = a.zeros[rr];
    st.zf = (float)st.zero;
    st.e2 = 0.f;
    lds_floats ub = (lds_floats)ubs + (threadIdx.x & 15);
    request_first<FactorState<WT>>(st, ub, std::make_integer_sequence<int, ustream::RING>{});
    st.active = active;
    st.edst = a.D + rr * a.ldd;
    // Codes go straight to their place when the block is whole and the row's 128 bytes are 16-byte aligned; otherwise
    // (last, short block; odd leading dimension) to a 128-byte slot of the row in the scratch area `cstage`, and the
    // valid ones are copied out below.
    const bool direct = a.nbk == QB && ((reinterpret_cast<uintptr_t>(a.codes + rr * a.ldc + a.j0) & 15) == 0);
    st.cdst = direct ? a.codes + rr * a.ldc + a.j0 : a.cstage + rr * QB;
    factor_columns<WT>(st, ub, maxq, std::make_integer_sequence<int, QB>{});
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

// One workgroup per row: the per-row grid from the original weights, and the row of accumulators cleared.
template <typename T>
__global__ __launch_bounds__(256) void prepare_rows_rf_kernel(const T* W, int64_t ldw, int64_t n, float* S, int64_t lds_,
                                                              int want_grid, int grid, float maxq, float* scales, int32_t* zeros) {
    const int64_t row = blockIdx.x;
    float lo = INFINITY, hi = -INFINITY, am = 0.f;
    if (!want_grid) {                                       // grouped grids are taken block by block, from the current weights
        for (int64_t k = threadIdx.x; k < n; k += 256) S[row * lds_ + k] = 0.f;
        return;
    }
    for (int64_t k = threadIdx.x; k < n; k += 256) {
        const float v = to_f32<T>(W[row * ldw + k]);
        S[row * lds_ + k] = 0.f;
        lo = fminf(lo, v); hi = fmaxf(hi, v); am = fmaxf(am, fabsf(v));
    }
    __shared__ float slo[256], shi[256], sam[256];
    slo[threadIdx.x] = lo; shi[threadIdx.x] = hi; sam[threadIdx.x] = am;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            slo[threadIdx.x] = fminf(slo[threadIdx.x], slo[threadIdx.x + w]);
            shi[threadIdx.x] = fmaxf(shi[threadIdx.x], shi[threadIdx.x + w]);
            sam[threadIdx.x] = fmaxf(sam[threadIdx.x], sam[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float sc; int zr;
        grid_from_range(grid, maxq, slo[0], shi[0], sam[0], sc, zr);
        scales[row] = sc; zeros[row] = zr;
    }
}

// Wq = scale * (code - zero)
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* codes, int64_t ldc, const float* scales, const int32_t* zeros,
                                                      int64_t ngroups, int64_t gsize, int64_t n, float* Wq, int64_t ldq) {
    const int64_t row = blockIdx.x;
    for (int64_t k = threadIdx.x; k < n; k += 256) {
        const int64_t gi = k / gsize;
        const float sc = scales[row * ngroups + gi];
        const float zf = (float)zeros[row * ngroups + gi];
        Wq[row * ldq + k] = sc * ((float)codes[row * ldc + k] - zf);
    }
}

static bool group_supported(int64_t group) {
    if (group == 0) return true;
    if (group < 0) return false;
    if (group % QB == 0) return true;
    return group == 8 || group == 16 || group == 32 || group == 64;
}

// The factor form takes one grid per row, or groups that lie inside a block and are wide enough for the walk to be
// worth instantiating (32, 64, 128).
static bool factor_form_group_supported(int64_t group) { return group == 0 || group == 32 || group == 64 || group == 128; }

constexpr int QOB = 1024;   // outer block: trailing updates beyond it are deferred and applied as one rank-1024 GEMM
static_assert(QOB == SPLIT_K, "the split products take exactly one outer block as K");

// The deferred rank-1024 updates go through the split-operand kernel (bf16 matrix cores, 256 x 256 tiles, one per
// workgroup) when rows and columns come in whole tiles and the launch fills the chip well (split_pays).
static bool split_shapes_ok(int64_t r, int64_t n) { return r >= 256 && r % 256 == 0 && n % 256 == 0 && n >= 2 * QOB; }

struct QuantWs { size_t wk, e, cs, ub, rt, pa, pb, pr, total; int64_t ldk; bool split; };
static QuantWs quant_ws_layout(int64_t r, int64_t n, int64_t group) {
    QuantWs l;
    l.ldk = (int64_t)round_up((size_t)std::max<int64_t>(n, 1), 4);
    l.wk = 0;
    size_t off = round_up((size_t)std::max<int64_t>(r, 1) * l.ldk * sizeof(float), 256);
    l.e = off; off += 2 * round_up((size_t)std::max<int64_t>(r, 1) * QOB * sizeof(float), 256);   // two error panels (look-ahead)
    l.cs = off; off += round_up((size_t)std::max<int64_t>(r, 1) * QB, 256);                        // codes of a block that cannot be stored in place
    l.ub = off; off += round_up((size_t)ceil_div(std::max<int64_t>(n, 1), QB) * QB * QB * sizeof(float), 256);   // factor form with groups: every U_bb
    l.rt = off;                                                                                       // ... and R with its column blocks scaled by them
    if (group != 0 && factor_form_group_supported(group)) off += round_up((size_t)std::max<int64_t>(n, 1) * l.ldk * sizeof(float), 256);
    // split products (gemm_split.hip): the bf16 pieces of an error panel, of the next outer block's rows of U and of all rows beyond
    l.split = split_shapes_ok(r, n);
    l.pa = l.pb = l.pr = off;
    if (l.split) {
        l.pa = off; off += round_up(split_planes_bytes(r), 256);
        l.pb = off; off += round_up(split_planes_bytes(QOB), 256);
        l.pr = off; off += round_up(split_planes_bytes(n), 256);
    }
    l.total = off + 256;
    return l;
}

}  // namespace gptq

using namespace gptq;

extern "C" int gptq_trailing_update(float* W, int64_t ldw, const float* E, int64_t lde, const float* U, int64_t ldu,
                                    int64_t r, int64_t ncols, int64_t k, void* stream) {
    if (r < 0 || ncols < 0 || k < 0) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update: negative size");
    if (r == 0 || ncols == 0 || k == 0) return GPTQ_OK;
    if (!W || !E || !U) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update: null pointer");
    if (ldw < ncols || lde < k || ldu < ncols) return fail(GPTQ_ERR_INVALID_ARG, "trailing_update: leading dimension smaller than the row length");
    if (!aligned(W, 16) || !aligned(E, 16) || !aligned(U, 16) || ldw % 4 || lde % 4 || ldu % 4)
        return fail(GPTQ_ERR_INVALID_ARG, "trailing_update: W, E and U must be 16-byte aligned with leading dimensions that are multiples of 4");
    GemmF32 g{};
    g.A = E; g.lda = lde; g.B = U; g.ldb = ldu; g.C = W; g.ldc = ldw;
    g.M = r; g.N = ncols; g.K = k; g.alpha = -1.f; g.b_is_nk = false; g.overwrite = false;
    return launch_gemm_f32(g, static_cast<hipStream_t>(stream));
}

extern "C" size_t gptq_quantize_layer_workspace_bytes(int64_t r, int64_t n, int block, int64_t group) {
    (void)block;
    if (r < 0 || n < 0) return 0;
    return quant_ws_layout(r, n, group).total;
}

// Both forms of Alg. 1 share validation, blocking and look-ahead.  rf = false: `U` is Cholesky((H + lambda I)^-1)^T,
// the working weights are updated (W -= E U).  rf = true: `U` is R with H + lambda I = R R^T, the accumulators are
// updated (S += D R) and the weights are read from the caller's W as they are (one grid per row only).
static int alg1_run(bool rf, const void* W, int wdtype, int64_t ldw, int64_t r, int64_t n,
                    const float* U, int64_t ldu,
                    int bits, int grid, int block, int64_t group,
                    uint8_t* codes, int64_t ldc, float* scales, int32_t* zeros,
                    float* Wq, int64_t ldq, double* half_E2_rows,
                    void* ws, size_t ws_bytes, void* stream) {
    if (r < 0 || n < 0) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: negative size");
    if (grid != GPTQ_GRID_MINMAX && grid != GPTQ_GRID_TERNARY) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: unknown grid %d", grid);
    if (grid == GPTQ_GRID_MINMAX && (bits < 2 || bits > 4)) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: bits must be 2, 3 or 4 (got %d)", bits);
    if (wdtype != GPTQ_F16 && wdtype != GPTQ_BF16 && wdtype != GPTQ_F32) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: unknown wdtype %d", wdtype);
    if (block <= 0) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: block must be positive");
    if (block != QB) return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer: only block = 128 is built (got %d)", block);
    if (group < 0) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: negative group");
    if (group > 0 && n % group) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: n must be a multiple of the group size");
    if (group > 0 && (QB % group) && (group % QB)) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: a group must not straddle a block end (need 128 %% g == 0 or g %% 128 == 0)");
    if (!group_supported(group)) return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer: group size %lld not built (8, 16, 32, 64 or a multiple of 128)", (long long)group);
    if (rf && !factor_form_group_supported(group))
        return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer_from_factor: one grid per row or groups of 32, 64 or 128 columns (got %lld); a group's grid "
                                          "is taken from the current weights, which this form rebuilds one block at a time: use "
                                          "gptq_damp_cholesky_inverse + gptq_quantize_layer", (long long)group);
    if (r == 0 || n == 0) return GPTQ_OK;
    if (!W || !U || !codes || !scales || !zeros) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: null pointer");
    if (ldw < n || ldu < n || ldc < n || (Wq && ldq < n)) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: leading dimension smaller than n");
    if (!aligned(U, 16) || ldu % 4) return fail(GPTQ_ERR_INVALID_ARG, "quantize_layer: U must be 16-byte aligned with ldu %% 4 == 0");
    const QuantWs lay = quant_ws_layout(r, n, group);
    if (!ws || !aligned(ws, 256) || ws_bytes < lay.total) return fail(GPTQ_ERR_WORKSPACE, "quantize_layer: workspace missing, misaligned or too small");
    if (r > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "quantize_layer: too many rows");

    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    float* Wk = reinterpret_cast<float*>(base + lay.wk);
    float* Ebuf[2] = {reinterpret_cast<float*>(base + lay.e),
                      reinterpret_cast<float*>(base + lay.e + round_up((size_t)r * QOB * sizeof(float), 256))};
    const int maxq = (grid == GPTQ_GRID_TERNARY) ? 2 : ((1 << bits) - 1);
    const int64_t ngroups = group ? n / group : 1;
    const int want_grid = group == 0;

    if (rf) {
        switch (wdtype) {
            case GPTQ_F16:
                hipLaunchKernelGGL(prepare_rows_rf_kernel<_Float16>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const _Float16*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
                break;
            case GPTQ_BF16:
                hipLaunchKernelGGL(prepare_rows_rf_kernel<__bf16>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const __bf16*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
                break;
            default:
                hipLaunchKernelGGL(prepare_rows_rf_kernel<float>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const float*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
        }
    } else
    switch (wdtype) {
        case GPTQ_F16:
            hipLaunchKernelGGL(prepare_rows_kernel<_Float16>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const _Float16*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
            break;
        case GPTQ_BF16:
            hipLaunchKernelGGL(prepare_rows_kernel<__bf16>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const __bf16*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
            break;
        default:
            hipLaunchKernelGGL(prepare_rows_kernel<float>, dim3((unsigned)r), dim3(256), 0, s, static_cast<const float*>(W), ldw, n, Wk, lay.ldk, want_grid, grid, (float)maxq, scales, zeros);
    }
    GPTQ_LAUNCH_CHECK();
    const bool hybrid = rf && group != 0;
    float* Ub = reinterpret_cast<float*>(base + lay.ub);
    // The matrix the deferred updates multiply with: U, R, or -- factor form with groups -- Rt = R with every column block
    // scaled by the inverse of its diagonal block (made here, once), so that the accumulators of a block hold s R_bb^-1.
    const float* Bm = U;
    int64_t ldb = ldu;
    if (hybrid) {
        float* Rt = reinterpret_cast<float*>(base + lay.rt);
        if (int rc = launch_invert_diag_blocks(U, ldu, n, Ub, s)) return rc;
        if (int rc = launch_scale_column_blocks(U, ldu, n, Ub, Rt, lay.ldk, s)) return rc;
        Bm = Rt; ldb = lay.ldk;
    }

    unsigned char* Pa = reinterpret_cast<unsigned char*>(base + lay.pa);
    unsigned char* Pb = reinterpret_cast<unsigned char*>(base + lay.pb);
    unsigned char* Pr = reinterpret_cast<unsigned char*>(base + lay.pr);
    const unsigned qblocks = (unsigned)ceil_div(r, 256);
    // Lazy batching at two levels (Section 3, Step 2 applied twice): inside an outer block of 1024 columns
    // each 128-column block updates only the rest of the outer block (rank 128); the columns beyond it
    // get one rank-1024 update per outer block.  Same sums as Alg. 1, associated differently.
    // A group grid must see fully updated weights at its first column, so an outer block may only end
    // where a group ends: groups that neither divide 1024 nor are multiples of it fall back to one level.
    const int64_t ob = (group >= QB && (QOB % group) && (group % QOB)) ? QB : QOB;
    // Look-ahead: after an outer block is quantized, the columns of the next outer block are updated first, on
    // the caller's stream, which goes straight on to quantize them (short, serial kernels); all columns
    // beyond are updated on the helper stream meanwhile.  The two updates and the next block's kernels touch
    // disjoint columns of the weights; the error panel E alternates between two buffers because the helper's
    // GEMM still reads one while the next block fills the other.
    TwoStreams ts;
    if (int rc = ts.open(s, true)) return rc;
    hipStream_t s2 = ts.side;
    hipEvent_t rest_done = nullptr;         // the helper stream's last trailing update, if one is pending
    int eb = 0;
    for (int64_t o0 = 0; o0 < n; o0 += ob, eb ^= 1) {
        const int64_t o1 = std::min<int64_t>(o0 + ob, n);
        float* E = Ebuf[eb];
        for (int64_t j0 = o0; j0 < o1; j0 += QB) {
            const int nbk = (int)std::min<int64_t>(QB, n - j0);
            const int64_t j1 = j0 + nbk;
            if (group > QB && j0 % group == 0) {
                // The grid is taken from all columns of the group as they stand now.  Those beyond this outer
                // block are kept current by the helper stream: its last update has to be in.
                if (j0 + group > o1) { if (int rc = ts.wait(s, rest_done)) return rc; }
                hipLaunchKernelGGL(group_grid_kernel, dim3((unsigned)r), dim3(64), 0, s, (const float*)Wk, lay.ldk, j0, group, grid, (float)maxq, scales, zeros, ngroups, j0 / group);
                GPTQ_LAUNCH_CHECK();
            }
            if (hybrid) {
                HybridArgs h{};
                h.W = W; h.ldw = ldw; h.T = Wk + j0; h.ldt = lay.ldk; h.Ub = Ub + (j0 / QB) * QB * QB; h.r = r; h.n = n; h.j0 = j0; h.nbk = nbk;
                h.grid = grid; h.maxq = maxq; h.scales = scales; h.zeros = zeros; h.ngroups = ngroups;
                h.codes = codes; h.ldc = ldc; h.cstage = reinterpret_cast<uint8_t*>(base + lay.cs);
                h.D = E + (j0 - o0); h.ldd = QOB; h.half_e2 = half_E2_rows; h.first_block = (j0 == 0);
                if (int rc = launch_quant_block_hybrid(group, wdtype, qblocks, h, s)) return rc;
            } else if (rf) {
                FactorArgs f{};
                f.W = W; f.ldw = ldw; f.S = Wk; f.lds_ = lay.ldk; f.R = U; f.ldr = ldu; f.r = r; f.n = n; f.j0 = j0; f.nbk = nbk;
                f.maxq = maxq; f.scales = scales; f.zeros = zeros; f.codes = codes; f.ldc = ldc;
                f.cstage = reinterpret_cast<uint8_t*>(base + lay.cs);
                f.D = E + (j0 - o0); f.ldd = QOB; f.half_e2 = half_E2_rows; f.first_block = (j0 == 0);
                switch (wdtype) {
                    case GPTQ_F16:  hipLaunchKernelGGL(quant_block_rf_kernel<_Float16>, dim3(qblocks), dim3(256), 0, s, f); break;
                    case GPTQ_BF16: hipLaunchKernelGGL(quant_block_rf_kernel<__bf16>,  dim3(qblocks), dim3(256), 0, s, f); break;
                    default:        hipLaunchKernelGGL(quant_block_rf_kernel<float>,   dim3(qblocks), dim3(256), 0, s, f); break;
                }
            } else {
            QuantArgs a{};
            a.Wk = Wk; a.ldk = lay.ldk; a.U = U; a.ldu = ldu; a.r = r; a.n = n; a.j0 = j0; a.nbk = nbk; a.grid = grid; a.maxq = maxq;
            a.scales = scales; a.zeros = zeros; a.ngroups = ngroups; a.group = group;
            a.codes = codes; a.ldc = ldc; a.E = E + (j0 - o0); a.lde = QOB; a.half_e2 = half_E2_rows; a.first_block = (j0 == 0);
            const int G = (group > 0 && group <= QB) ? (int)group : 0;
            switch (G) {
                case 0:  hipLaunchKernelGGL(quant_block_kernel<0>,  dim3(qblocks), dim3(256), 0, s, a); break;
                case 128: hipLaunchKernelGGL(quant_block_kernel<128>, dim3(qblocks), dim3(256), 0, s, a); break;
                case 8:  hipLaunchKernelGGL(quant_block_kernel<8>,  dim3(qblocks), dim3(256), 0, s, a); break;
                case 16: hipLaunchKernelGGL(quant_block_kernel<16>, dim3(qblocks), dim3(256), 0, s, a); break;
                case 32: hipLaunchKernelGGL(quant_block_kernel<32>, dim3(qblocks), dim3(256), 0, s, a); break;
                default: hipLaunchKernelGGL(quant_block_kernel<64>, dim3(qblocks), dim3(256), 0, s, a); break;
            }
            }
            GPTQ_LAUNCH_CHECK();
            if (j1 < o1) {
                // Inside the outer block the updates are batched once more, in pairs of blocks: after the first block of a
                // pair only the second block's columns are brought up to date (rank 128, 128 columns wide); after the second,
                // everything beyond the pair gets both blocks' contributions in one rank-256 product.  Same sums, associated
                // differently: 16 instead of 28 block columns of the accumulators are read and written per outer block, and
                // the wide products have twice the K.  Where the layer has many rows these products are what the step costs
                // (Alg. 1 on a 49152 x 12288 layer 52.5 -> 50.6 ms; neutral at 12288 rows; the same batching in the
                // factorisation made its chain slower, 11.6 -> 11.8 ms at n = 12288, and is not used there; a full binary
                // tree of batches -- rank 512 after the fourth block -- gained 0.4 ms more at 49152 rows and lost 1.7 ms on
                // the 12288 x 49152 layer, whose chain then waits for longer products).
                // A group grid that starts at the second block of a pair and reaches beyond it (a group of 384 columns) would
                // see columns that still lack the first block's contribution: such layers keep one update per block.
                const bool pairs = group <= QB || group % (2 * QB) == 0;
                const int64_t idx = (j0 - o0) / QB;
                GemmF32 g{};
                g.lda = QOB; g.ldb = ldb; g.ldc = lay.ldk; g.M = r; g.alpha = rf ? 1.f : -1.f; g.b_is_nk = false; g.overwrite = false;
                if (!pairs) {
                    g.A = E + (j0 - o0); g.B = Bm + j0 * ldb + j1; g.C = Wk + j1; g.N = o1 - j1; g.K = nbk;
                } else if (idx % 2 == 0) {
                    g.A = E + (j0 - o0); g.B = Bm + j0 * ldb + j1; g.C = Wk + j1; g.N = std::min<int64_t>(QB, o1 - j1); g.K = nbk;
                } else {
                    g.A = E + (j0 - QB - o0); g.B = Bm + (j0 - QB) * ldb + j1; g.C = Wk + j1; g.N = o1 - j1; g.K = QB + nbk;
                }
                const int rc = launch_gemm_f32(g, s);
                if (rc) return rc;
            }
        }
        if (o1 < n) {
            const int64_t o2 = std::min<int64_t>(o1 + ob, n);
            hipEvent_t quantized = nullptr;
            if (int rc = ts.mark(s, &quantized)) return rc;
            if (int rc = ts.wait(s, rest_done)) return rc;      // it wrote the columns from o1 on
            rest_done = nullptr;
            const float alpha = rf ? 1.f : -1.f;
            const bool full = lay.split && ob == QOB && o1 - o0 == QOB;
            const bool split_strip = full && o2 - o1 == QOB && split_pays((r / 256) * (QOB / 256));
            const bool split_rest = full && o2 < n && split_pays((r / 256) * ((n - o2) / 256));
            SplitGemm sg{};
            sg.A_planes = Pa; sg.A_zero = split_zero_block(Pa, r); sg.a_panel0 = 0;
            sg.ldc = lay.ldk; sg.alpha = alpha; sg.tiles_m = (int)(r / 256);
            GemmF32 g{};
            g.A = E; g.lda = QOB; g.B = Bm + o0 * ldb + o1; g.ldb = ldb; g.C = Wk + o1; g.ldc = lay.ldk;
            g.M = r; g.N = o2 - o1; g.K = o1 - o0; g.alpha = alpha; g.b_is_nk = false; g.overwrite = false;
            if (split_strip) {
                // the pieces of the error panel are made here, for both parts (the helper stream's last reader of the
                // buffer is what the wait above was for); those of U's rows for the next outer block's columns as well
                if (int rc = launch_split_rows(E, QOB, r, Pa, s)) return rc;
                if (int rc = launch_split_cols(Bm + o0 * ldb + o1, ldb, QOB, Pb, s)) return rc;
                if (int rc = ts.mark(s, &quantized)) return rc;
                sg.B_planes = Pb; sg.B_zero = split_zero_block(Pb, QOB); sg.b_panel0 = 0;
                sg.C = Wk + o1; sg.tiles_n = QOB / 256;
                if (int rc = launch_gemm_split(sg, s)) return rc;
            } else {
                if (int rc = launch_gemm_f32(g, s)) return rc;
            }
            if (o2 < n) {
                if (split_rest) {
                    // U's rows for all columns beyond depend on nothing of this outer block: they are split before the helper
                    // stream waits for it (the buffer's last reader, the previous rest update, precedes this on the stream)
                    if (int rc = launch_split_cols(Bm + o0 * ldb + o2, ldb, n - o2, Pr, s2)) return rc;
                }
                if (int rc = ts.wait(s2, quantized)) return rc;
                if (split_rest) {
                    if (!split_strip) { if (int rc = launch_split_rows(E, QOB, r, Pa, s2)) return rc; }
                    sg.B_planes = Pr; sg.B_zero = split_zero_block(Pr, n - o2); sg.b_panel0 = 0;
                    sg.C = Wk + o2; sg.tiles_n = (int)((n - o2) / 256);
                    if (int rc = launch_gemm_split(sg, s2)) return rc;
                } else {
                    g.B = Bm + o0 * ldb + o2; g.C = Wk + o2; g.N = n - o2;
                    if (int rc = launch_gemm_f32(g, s2)) return rc;
                }
                if (int rc = ts.mark(s2, &rest_done)) return rc;
            }
        }
    }
    if (Wq) {
        hipLaunchKernelGGL(dequant_kernel, dim3((unsigned)r), dim3(256), 0, s, (const uint8_t*)codes, ldc, (const float*)scales, (const int32_t*)zeros,
                           ngroups, group ? group : n, n, Wq, ldq);
        GPTQ_LAUNCH_CHECK();
    }
    return GPTQ_OK;
}

extern "C" int gptq_quantize_layer(const void* W, int wdtype, int64_t ldw, int64_t r, int64_t n,
                                   const float* U, int64_t ldu,
                                   int bits, int grid, int block, int64_t group,
                                   uint8_t* codes, int64_t ldc, float* scales, int32_t* zeros,
                                   float* Wq, int64_t ldq, double* half_E2_rows,
                                   void* ws, size_t ws_bytes, void* stream) {
    return alg1_run(false, W, wdtype, ldw, r, n, U, ldu, bits, grid, block, group, codes, ldc, scales, zeros, Wq, ldq,
                    half_E2_rows, ws, ws_bytes, stream);
}

extern "C" int gptq_quantize_layer_from_factor_supports(int64_t group) { return factor_form_group_supported(group) ? 1 : 0; }

extern "C" int gptq_quantize_layer_from_factor(const void* W, int wdtype, int64_t ldw, int64_t r, int64_t n,
                                               const float* R, int64_t ldr,
                                               int bits, int grid, int block, int64_t group,
                                               uint8_t* codes, int64_t ldc, float* scales, int32_t* zeros,
                                               float* Wq, int64_t ldq, double* half_E2_rows,
                                               void* ws, size_t ws_bytes, void* stream) {
    return alg1_run(true, W, wdtype, ldw, r, n, R, ldr, bits, grid, block, group, codes, ldc, scales, zeros, Wq, ldq,
                    half_E2_rows, ws, ws_bytes, stream);
}
