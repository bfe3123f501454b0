// Device code shared by the translation units of step 3 (Algorithm 1): the conversion helpers, the grid of
// Section 4 from a range of weights, and the machinery with which a lane walks the 128 columns of a block -- the
// stream of a 128 x 128 triangular block through LDS and the DPP row broadcast, the rank-1 update of a column.
#pragma once
#include "common.h"

#include <utility>

namespace gptq {

constexpr int QB = 128;

// ---- W (f16 / bf16 / f32) -> float32 working copy; optionally the per-row grid from the original row.
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<_Float16>(_Float16 v) { return (float)v; }
template <> __device__ __forceinline__ float to_f32<__bf16>(__bf16 v) { return (float)v; }

__device__ __forceinline__ void grid_from_range(int grid, float maxq, float lo, float hi, float amax, float& scale, int& zero) {
    if (grid == GPTQ_GRID_TERNARY) {
        scale = (amax == 0.f) ? 1.f : amax;
        zero = 1;
    } else {
        lo = fminf(lo, 0.f);
        hi = fmaxf(hi, 0.f);
        if (hi == lo) { scale = 1.f; zero = 0; }
        else {
            scale = (hi - lo) / maxq;
            zero = (int)rintf(-lo / scale);
        }
    }
}

// ---- the stream of U values ------------------------------------------------------------------------------
// Row j of the block of U is needed from the aligned chunk of 16 floats that holds column j: the diagonal
// element and the elements right of it.  A chunk sits in ONE register: lane l holds element l % 16 (the same
// 16 values in each of the wavefront's four rows of 16 lanes), and the multiply-add that needs element c reads
// it from lane c of its own row through the DPP row broadcast -- v_fmac_f32_dpp ... row_newbcast:c -- so a value
// of U reaches all 64 lanes inside the instruction that uses it.  (Reading each value into every lane with
// 16-byte LDS reads cost as many issue cycles per value as the multiply-add itself.)
// All rows' chunks, in the order of their use, form one stream; it is read from LDS through a ring of RING
// registers: the chunk at stream position t + RING is requested right after the one at position t has been used,
// so a request runs well over a thousand cycles ahead of its use, also across the serial arithmetic at a column.
// Rows, chunks and ring slots are template parameters: every register index is a constant by construction.
namespace ustream {
constexpr int RING = 8;
constexpr int CHUNK = 16;
constexpr int first_chunk(int j) { return j / CHUNK; }
constexpr int chunks(int j) { return QB / CHUNK - first_chunk(j); }
constexpr int start(int j) { int s = 0; for (int i = 0; i < j; ++i) s += chunks(i); return s; }
constexpr int TOTAL = start(QB);
constexpr int row_at(int t) { int j = 0; while (t >= chunks(j)) { t -= chunks(j); ++j; } return j; }
}  // namespace ustream

typedef const __attribute__((address_space(3))) float* lds_floats;
typedef const volatile __attribute__((address_space(3))) float* lds_floats_ordered;

template <typename WT> struct WeightRegs {                  // float32 weights: one register each
    float v[QB];
    template <int J> __device__ __forceinline__ float get() const { return v[J]; }
};
template <> struct WeightRegs<_Float16> {                    // 16-bit weights stay packed two to a register
    uint32_t v[QB / 2];
    template <int J> __device__ __forceinline__ float get() const {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(v[J / 2] >> (16 * (J & 1))));
    }
};
template <> struct WeightRegs<__bf16> {
    uint32_t v[QB / 2];
    template <int J> __device__ __forceinline__ float get() const {
        return __builtin_bit_cast(float, (J & 1) ? (v[J / 2] & 0xffff0000u) : (v[J / 2] << 16));
    }
};


// Volatile on purpose: volatile accesses and volatile asm statements (the multiply-adds below) keep their
// program order, which is what places each request RING chunks ahead of its use.  An ordinary load has no such
// order: with the whole column loop one straight line, the compiler either hoists all requests to the top or
// sinks each one down to its use and then waits for it.  `ubl` is the block in LDS offset by lane % 16.
template <int T, class St>
__device__ __forceinline__ void request_chunk(St& st, lds_floats ubl) {
    if constexpr (T < ustream::TOTAL) {
        constexpr int j = ustream::row_at(T), q = ustream::first_chunk(j) + (T - ustream::start(j));
        st.ring[T % ustream::RING] = *static_cast<lds_floats_ordered>(ubl + j * QB + ustream::CHUNK * q);
    }
}

template <class St, int... T>
__device__ __forceinline__ void request_first(St& st, lds_floats ubl, std::integer_sequence<int, T...>) {
    (request_chunk<T>(st, ubl), ...);
}

// w[k] += ne * (element C of the chunk in `u`), for all lanes.  The s_nop covers the two wait states a DPP read
// needs after a vector-ALU write of the same register, should the compiler ever have moved the chunk there.
template <int C, bool FIRST>
__device__ __forceinline__ void fma_bcast(float& w, float u, float ne) {
    if constexpr (FIRST)
        asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(w) : "v"(u), "v"(ne), "n"(C));
    else
        asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(w) : "v"(u), "v"(ne), "n"(C));
}

template <int J, int K0, class St, int... C>
__device__ __forceinline__ void update_chunk_columns(St& st, float u, float ne, std::integer_sequence<int, C...>) {
    // columns K0 + C right of J; the first one issued carries the s_nop
    constexpr int first = (J >= K0) ? J - K0 + 1 : 0;
    ((K0 + C > J ? fma_bcast<C, C == first>(st.acc()[K0 + C], u, ne) : (void)0), ...);
}

// w[k] -= e * U[J][k] for the columns of chunk Q right of J, then the request that refills the slot
template <int J, int Q, class St>
__device__ __forceinline__ void update_chunk(St& st, lds_floats ubl, float ne) {
    constexpr int t = ustream::start(J) + Q, k0 = ustream::CHUNK * (ustream::first_chunk(J) + Q);
    update_chunk_columns<J, k0>(st, st.ring[t % ustream::RING], ne, std::make_integer_sequence<int, ustream::CHUNK>{});
    request_chunk<t + ustream::RING>(st, ubl);
}

template <int J, class St, int... Q>
__device__ __forceinline__ void update_row(St& st, lds_floats ubl, float ne, std::integer_sequence<int, Q...>) {
    (update_chunk<J, Q>(st, ubl, ne), ...);
}

// The 128 x 128 diagonal block of an upper-triangular matrix M (U, or the factor R) into LDS:
// ubs[j][k] = M[j0+j][j0+k] for k >= j, zero below the diagonal, identity outside the matrix.  The whole workgroup
// (256 threads) calls it: 16 independent 16-byte loads per thread (in PARTS passes of 16 / PARTS, for callers short
// of registers), then one barrier.
template <int PARTS = 1>
__device__ __forceinline__ void stage_diag_block(float* ubs, const float* M, int64_t ldm, int64_t j0, int64_t n) {
    const int tid = threadIdx.x;
    constexpr int PER = 16 / PARTS;
#pragma unroll
    for (int part = 0; part < PARTS; ++part) {
    float4 in[PER];
#pragma unroll
    for (int tt = 0; tt < PER; ++tt) {
        const int t = part * PER + tt;
        const int q = tid + 256 * t, j = q >> 5, k = (q & 31) * 4;
        const int64_t gj = j0 + j, gk = j0 + k;
        const float* src = M + gj * ldm + gk;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gj < n && gk + 4 <= n) v = *reinterpret_cast<const float4*>(src);
        else if (gj < n && gk < n) { v.x = src[0]; if (gk + 1 < n) v.y = src[1]; if (gk + 2 < n) v.z = src[2]; }
        in[tt] = v;
    }
#pragma unroll
    for (int tt = 0; tt < PER; ++tt) {
        const int t = part * PER + tt;
        const int q = tid + 256 * t, j = q >> 5, k = (q & 31) * 4;
        const int64_t gj = j0 + j, gk = j0 + k;
        float e[4] = {in[tt].x, in[tt].y, in[tt].z, in[tt].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool inside = gj < n && gk + c < n;
            e[c] = inside ? (k + c >= j ? e[c] : 0.f) : (k + c == j ? 1.f : 0.f);
        }
        *reinterpret_cast<float4*>(&ubs[j * QB + k]) = make_float4(e[0], e[1], e[2], e[3]);
    }
    }
    __syncthreads();
}

// ---- the factor form with grids taken inside a block: arguments and launchers (quantize_groups.hip) ----
struct HybridArgs {
    const void* W; int64_t ldw;     // original weights, type WT
    const float* T; int64_t ldt;    // this block's 128 columns of the accumulators, which hold S[:, block] U_bb
    const float* Ub;                // U_bb, dense 128 x 128 (identity outside a short last block)
    int64_t r, n, j0; int nbk;
    int grid; int maxq;
    float* scales; int32_t* zeros; int64_t ngroups;
    uint8_t* codes; int64_t ldc;
    uint8_t* cstage;
    float* D; int64_t ldd;
    double* half_e2;
    int first_block;
};

// Launches the walk of one block for group in {32, 64, 128} and wdtype in {GPTQ_F16, GPTQ_BF16, GPTQ_F32}.
int launch_quant_block_hybrid(int64_t group, int wdtype, unsigned workgroups, const HybridArgs& h, hipStream_t s);
// Ub[b] = R_bb^-1 for every 128 x 128 diagonal block of R (dense, identity outside a short last block).
int launch_invert_diag_blocks(const float* R, int64_t ldr, int64_t n, float* Ub, hipStream_t s);
// Rt[0:j0, block] = R[0:j0, block] U_bb for every column block (the part above the diagonal blocks; the rest of Rt is
// not written).
int launch_scale_column_blocks(const float* R, int64_t ldr, int64_t n, const float* Ub, float* Rt, int64_t ldt, hipStream_t s);

}  // namespace gptq
