// Consumers of the packed format (Section 4, "Practical Speedups", and the appendix on the benchmarking
// setup): the full-matrix decompression used before a large-batch product, and the quantized-matrix times
// full-precision-vector product of batch-1 generation, which dequantizes weights as it reads them and does
// not quantize the vector.  Both are bound by HBM: the packed words are read once.
//
// Layout (same as pack.hip): per row, code k occupies bits [k*b, (k+1)*b) of a little-endian stream of uint32
// words; 32 codes are exactly b words.  A weight is scale * (code - zero) with the scale and zero point of its
// row (group == 0) or of its row's group k / group.
#include "common.h"

#include <hip/hip_fp16.h>

namespace gptq {

struct PackedArgs {
    const uint32_t* words; int64_t ldp;
    int64_t r, n, words_per_row;
    const float* scales; const int32_t* zeros;
    int64_t group, ngroups;      // group == 0: one grid per row (ngroups == 1)
    int gshift;                  // log2(group) if the group size is a power of two, else -1 (then columns are divided)
    int64_t rows_per_wg;         // matvec: rows a workgroup walks, a multiple of its row chunk
};

template <int BITS>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&w)[BITS], int i) {
    const int pos = i * BITS, wi = pos >> 5, off = pos & 31;
    uint32_t v = w[wi] >> off;
    if (off + BITS > 32) v |= w[(wi + 1) % BITS] << (32 - off);      // % only keeps the index in range for the compiler
    return v & ((1u << BITS) - 1u);
}

// ---- codes to halves without a conversion (used by both consumers) -------------------------------------------------
// With the exponent bits of 2^b or-ed in, a code sitting at mantissa bits [10-b, 10) of a half IS the float16 number
// 2^b + code.  Two codes whose bit positions differ by 16 (mod 32) sit at the same place of the two halves of a
// 32-bit word, so one shift puts both at [10-b, 10) / [26-b, 26) and one and-or masks them and sets both exponents:
//   b = 4: codes k and k+4 of a word;  b = 2: codes k and k+8 of a word;
//   b = 3: codes k and k+16 of the 96-bit group are 48 bits apart -- low half of one word, high half of another,
//          joined by one byte permute that serves four or five pairs; the two pairs whose codes straddle a
//          16-bit boundary (5, 21 and 10, 26) are cut out one code at a time.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

struct PairSpec { int lo_word, hi_word, rel, k_lo, k_hi; };      // lo_word < 0: cut the two codes out one at a time
template <int BITS> struct PairTable;
template <> struct PairTable<4> {
    static constexpr PairSpec at(int i) { return {i / 4, i / 4, 4 * (i % 4), 8 * (i / 4) + i % 4, 8 * (i / 4) + i % 4 + 4}; }
};
template <> struct PairTable<2> {
    static constexpr PairSpec at(int i) { return {i / 8, i / 8, 2 * (i % 8), 16 * (i / 8) + i % 8, 16 * (i / 8) + i % 8 + 8}; }
};
template <> struct PairTable<3> {
    static constexpr PairSpec at(int i) {
        if (i < 5) return {0, 1, 3 * i, i, i + 16};                                   // k = 0..4
        if (i < 9) return {2, 0, 3 * (i + 1) - 16, (i + 1) + 16, i + 1};              // k = 6..9
        if (i < 14) return {1, 2, 3 * (i + 2) - 32, i + 2, (i + 2) + 16};             // k = 11..15
        return i == 14 ? PairSpec{-1, -1, 0, 5, 21} : PairSpec{-1, -1, 0, 10, 26};
    }
};

__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t c) {
    uint32_t v;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(v) : "v"(a), "s"(mask), "v"(c));   // written out: the compiler spends two on it
    return v;
}

// 32 bits of the stream of words w[0..BITS] (w[BITS] = 0) starting at bit `from` (may be negative: shifted in zeros)
template <int BITS>
__device__ __forceinline__ uint32_t stream_bits(const uint32_t (&w)[BITS + 1], int from) {
    if (from < 0) return w[0] << (-from);
    const int wi = from >> 5, sh = from & 31;
    return sh ? __builtin_amdgcn_alignbit(w[wi + 1], w[wi], sh) : w[wi];
}


// The 32 codes of b words as 16 registers of two halves (2^b + code each); register i holds codes PairTable::at(i).k_lo
// (low half) and .k_hi (high half).  w[BITS] must be 0.
template <int BITS>
__device__ __forceinline__ void codes_as_half_pairs(const uint32_t (&w)[BITS + 1], uint32_t (&pr)[16]) {
    constexpr int WANT = 10 - BITS;
    constexpr uint32_t M = (1u << BITS) - 1u;
    constexpr uint32_t MASK_LO = M << WANT, MASK_HI = M << (16 + WANT), MASK = MASK_LO | MASK_HI;
    const uint32_t magic = 0x3C003C00u + (uint32_t)BITS * 0x04000400u;       // (2^b, 2^b) as two halves
    uint32_t joined[3] = {0u, 0u, 0u};
    if constexpr (BITS == 3) {
        joined[0] = __builtin_amdgcn_perm(w[1], w[0], 0x07060100u);      // low half of w0, high half of w1
        joined[1] = __builtin_amdgcn_perm(w[0], w[2], 0x07060100u);      // low half of w2, high half of w0
        joined[2] = __builtin_amdgcn_perm(w[2], w[1], 0x07060100u);      // low half of w1, high half of w2
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const PairSpec sp = PairTable<BITS>::at(i);
        if (sp.lo_word < 0) {
            const uint32_t ta = stream_bits<BITS>(w, BITS * sp.k_lo - WANT);
            const uint32_t tb = stream_bits<BITS>(w, BITS * sp.k_hi - (16 + WANT));
            pr[i] = and_or(tb, MASK_HI, and_or(ta, MASK_LO, magic));
        } else {
            uint32_t m;
            if (sp.lo_word == sp.hi_word) m = w[sp.lo_word];
            else m = joined[sp.lo_word == 0 ? 0 : (sp.lo_word == 2 ? 1 : 2)];
            const uint32_t t = sp.rel >= WANT ? (m >> (sp.rel - WANT)) : (m << (WANT - sp.rel));
            pr[i] = and_or(t, MASK, magic);
        }
    }
}

// ---- full-matrix decompression, the usual case (n a multiple of 8, one grid per 8 columns, 16-byte aligned rows) ----
// A workgroup walks along a row (then along every gridDim.x-th row after it), one thread per 8 codes per step:
// neighbouring lanes write neighbouring 16 bytes, so a store instruction of a wavefront covers 1 KB without a gap and a
// workgroup streams a whole row; lanes re-read words their neighbours also read (served by the vector cache).
// The 8 codes are 8 b consecutive bits of at most two words.  Or-ed into 0x6400 a code IS the half 1024 + code, so a
// pair of codes costs a shift and two and-ors, one packed subtraction of 1024 + zero leaves the exact integers
// code - zero, and each output is the float32 product with the scale, rounded to the output type.
template <int BITS, typename OT>
__global__ __launch_bounds__(256) void dequantize8_kernel(PackedArgs a, OT* __restrict__ out, int64_t ldo, int64_t octets_per_row) {
    constexpr uint32_t M = (1u << BITS) - 1u;
    constexpr int UN = 1;                       // octets per thread per step (256 apart; more in flight measured slower)
    for (int64_t row = blockIdx.x; row < a.r; row += gridDim.x) {
        const uint32_t* __restrict__ wrow = a.words + row * a.ldp;
        OT* orow = out + row * ldo;
        const float* srow = a.scales + row * a.ngroups;
        const int32_t* zrow = a.zeros + row * a.ngroups;
        for (int64_t oc0 = threadIdx.x; oc0 < octets_per_row; oc0 += 256 * UN) {
            uint32_t lo[UN], hi[UN];
            float sc[UN], zf[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t oc = oc0 + 256 * u;
                lo[u] = hi[u] = 0u; sc[u] = 0.f; zf[u] = 0.f;
                if (oc < octets_per_row) {
                    const int64_t bit0 = oc * 8 * BITS, wi = bit0 >> 5;
                    const int off = (int)(bit0 & 31);
                    lo[u] = wrow[wi];
                    if ((off + 8 * BITS > 32) && (wi + 1 < a.words_per_row)) hi[u] = wrow[wi + 1];
                    // column / group size without the 64-bit division (n < 2^31 columns are checked on the host)
                    const uint32_t col = (uint32_t)(oc * 8);
                    const uint32_t gcol = a.group == 0 ? 0u : (a.gshift >= 0 ? col >> a.gshift : col / (uint32_t)a.group);
                    sc[u] = srow[gcol];
                    zf[u] = (float)zrow[gcol];
                }
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int64_t oc = oc0 + 256 * u;
                if (oc >= octets_per_row) break;
                const int off = (int)((oc * 8 * BITS) & 31);
                const uint32_t bits8 = __builtin_amdgcn_alignbit(hi[u], lo[u], off);       // code i at bits [i*b, (i+1)*b)
                const _Float16 zh = (_Float16)(1024.f + zf[u]);                              // exact
                half2v z2; z2.x = zh; z2.y = zh;
                _Float16 d[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t t = bits8 >> (2 * i * BITS);                              // codes 2i and 2i+1 at the bottom
                    const uint32_t pair = and_or(t << (16 - BITS), M << 16, and_or(t, M, 0x64006400u));
                    const half2v v = __builtin_bit_cast(half2v, pair) - z2;
                    d[2 * i] = v.x; d[2 * i + 1] = v.y;
                }
                OT* dst = orow + oc * 8;
                if constexpr (sizeof(OT) == 2) {
                    union { uint4 u4; _Float16 h[8]; } pk;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        float prod = sc[u] * (float)d[i];       // the float32 product, rounded, and only then the half: the
                        asm volatile("" : "+v"(prod));          // two must not be fused into one mixed-precision instruction
                        pk.h[i] = (_Float16)prod;
                    }
                    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                    u32x4 v4; v4.x = pk.u4.x; v4.y = pk.u4.y; v4.z = pk.u4.z; v4.w = pk.u4.w;
                    __builtin_nontemporal_store(v4, reinterpret_cast<u32x4*>(dst));     // written once, not read again here
                } else {
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    f32x4 a4 = {sc[u] * (float)d[0], sc[u] * (float)d[1], sc[u] * (float)d[2], sc[u] * (float)d[3]};
                    f32x4 b4 = {sc[u] * (float)d[4], sc[u] * (float)d[5], sc[u] * (float)d[6], sc[u] * (float)d[7]};
                    __builtin_nontemporal_store(a4, reinterpret_cast<f32x4*>(dst));
                    __builtin_nontemporal_store(b4, reinterpret_cast<f32x4*>(dst) + 1);
                }
            }
        }
    }
}

// ---- full-matrix decompression, any shape: one thread per 8 codes = 8 consecutive outputs (one 16-byte store of halves) ---
// 8 codes are 8*b consecutive bits starting at a multiple of 8 bits: at most two words.  Neighbouring lanes
// write neighbouring 16 bytes, and re-read words their neighbours also read (served by the vector cache).
template <int BITS, typename OT>
__global__ __launch_bounds__(256) void dequantize_kernel(PackedArgs a, OT* out, int64_t ldo, int64_t octets_per_row) {
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= a.r * octets_per_row) return;
    const int64_t row = gid / octets_per_row, oc = gid % octets_per_row;
    const int64_t k0 = oc * 8;
    const int64_t bit0 = k0 * BITS, wi = bit0 >> 5;
    const int off = (int)(bit0 & 31);
    const uint32_t* p = a.words + row * a.ldp + wi;
    const uint64_t lo = p[0];
    const uint64_t hi = (off + 8 * BITS > 32 && wi + 1 < a.words_per_row) ? p[1] : 0u;
    const uint32_t bits8 = (uint32_t)(((hi << 32) | lo) >> off);        // the 8 codes, code i at bits [i*b, (i+1)*b)
    const bool one_grid = (a.group == 0) || (a.group % 8 == 0);
    const int64_t gbase = row * a.ngroups;
    float sc = 0.f, zf = 0.f;
    if (one_grid) {
        const int64_t gi = a.group ? k0 / a.group : 0;
        sc = a.scales[gbase + gi];
        zf = (float)a.zeros[gbase + gi];
    }
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (!one_grid && k0 + i < a.n) {
            const int64_t gi = (k0 + i) / a.group;
            sc = a.scales[gbase + gi];
            zf = (float)a.zeros[gbase + gi];
        }
        v[i] = sc * ((float)((bits8 >> (i * BITS)) & ((1u << BITS) - 1u)) - zf);
    }
    OT* dst = out + row * ldo + k0;
    if ((k0 + 8 <= a.n) && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
        if constexpr (sizeof(OT) == 2) {
            union { uint4 u; __half h[8]; } pk;
#pragma unroll
            for (int i = 0; i < 8; ++i) pk.h[i] = __float2half_rn(v[i]);
            *reinterpret_cast<uint4*>(dst) = pk.u;
        } else {
            reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
            reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (k0 + i < a.n) {
                if constexpr (sizeof(OT) == 2) dst[i] = __float2half_rn(v[i]);
                else dst[i] = v[i];
            }
    }
}

// ---- y = Q x, batch 1 -----------------------------------------------------------------------------------------
// A workgroup of 4 wavefronts owns MV_ROWS rows.  A wavefront walks every fourth 2048-column segment of those
// rows: a lane holds the 32 vector entries of its 32 columns in registers (read once per segment, shared by all
// the rows), reads b consecutive words per row -- a wavefront reads 64*b*4 contiguous bytes of a row -- and
// accumulates  scale * (sum code*x - zero * sum x)  in float32.  The lane sums of a row are reduced across the
// wavefront with DPP-style shuffles and across the four wavefronts through LDS.
constexpr int MV_ROWS = 4;
constexpr int MV_SEG = 64 * 32;

template <typename XT>
__device__ __forceinline__ void load_x32(const XT* x, int64_t k0, int64_t n, float (&xf)[32]) {
    if (k0 + 32 <= n && (reinterpret_cast<uintptr_t>(x + k0) & 15) == 0) {
        if constexpr (sizeof(XT) == 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                union { uint4 u; __half h[8]; } pk;
                pk.u = reinterpret_cast<const uint4*>(x + k0)[q];
#pragma unroll
                for (int i = 0; i < 8; ++i) xf[8 * q + i] = __half2float(pk.h[i]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float4 f = reinterpret_cast<const float4*>(x + k0)[q];
                xf[4 * q] = f.x; xf[4 * q + 1] = f.y; xf[4 * q + 2] = f.z; xf[4 * q + 3] = f.w;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            float v = 0.f;
            if (k0 + i < n) {
                if constexpr (sizeof(XT) == 2) v = __half2float(x[k0 + i]);
                else v = x[k0 + i];
            }
            xf[i] = v;                       // columns past n contribute nothing
        }
    }
}

// GSUB = number of grids inside a lane's 32 columns: 1 (one grid per row, or groups of a multiple of 32), 2 (16), 4 (8)
template <int BITS, int GSUB, typename XT>
__global__ __launch_bounds__(256) void matvec_kernel(PackedArgs a, const XT* x, float* y) {
    __shared__ float part[4][MV_ROWS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t nseg = (a.n + MV_SEG - 1) / MV_SEG;
    constexpr int GL = 32 / GSUB;            // columns per grid inside the lane's 32
    const int64_t row_end = min(((int64_t)blockIdx.x + 1) * a.rows_per_wg, a.r);
    for (int64_t row0 = (int64_t)blockIdx.x * a.rows_per_wg; row0 < row_end; row0 += MV_ROWS) {
    float acc[MV_ROWS];
#pragma unroll
    for (int rr = 0; rr < MV_ROWS; ++rr) acc[rr] = 0.f;
    for (int64_t s = wave; s < nseg; s += 4) {
        const int64_t k0 = s * MV_SEG + (int64_t)lane * 32;
        if (k0 >= a.n) continue;
        float xf[32];
        load_x32<XT>(x, k0, a.n, xf);
        float sx[GSUB];
#pragma unroll
        for (int j = 0; j < GSUB; ++j) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < GL; ++i) t += xf[j * GL + i];
            sx[j] = t;
        }
        const int64_t w0 = (k0 >> 5) * BITS;
        const int64_t g0 = a.group ? k0 / a.group : 0;
#pragma unroll
        for (int rr = 0; rr < MV_ROWS; ++rr) {
            const int64_t row = min(row0 + rr, a.r - 1);         // rows past r repeat the last one and are dropped below
            const uint32_t* p = a.words + row * a.ldp + w0;
            uint32_t w[BITS];
#pragma unroll
            for (int i = 0; i < BITS; ++i) w[i] = (w0 + i < a.words_per_row) ? p[i] : 0u;
#pragma unroll
            for (int j = 0; j < GSUB; ++j) {
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < GL; ++i) dot = fmaf((float)code_at<BITS>(w, j * GL + i), xf[j * GL + i], dot);
                const int64_t gi = row * a.ngroups + min(g0 + j, a.ngroups - 1);
                acc[rr] = fmaf(a.scales[gi], dot - (float)a.zeros[gi] * sx[j], acc[rr]);
            }
        }
    }
#pragma unroll
    for (int rr = 0; rr < MV_ROWS; ++rr) {
        float v = acc[rr];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        if (lane == 0) part[wave][rr] = v;
    }
    __syncthreads();
    if (threadIdx.x < MV_ROWS && row0 + threadIdx.x < a.r)
        y[row0 + threadIdx.x] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
    __syncthreads();
    }
}

// float16 vector, one grid per lane segment (one grid per row, or groups of a multiple of 32): two weights per
// v_dot2_f32_f16 on the pairs of halves 2^b + code made as above; the vector's halves are paired the same way once
// per segment.  The dot products accumulate sum (2^b + code) x in float32, and
// sum (code - zero) x = that - (2^b + zero) sum x;  the offset is of the size of the codes themselves, so the
// subtraction costs no accuracy worth naming.
constexpr int MV2_ROWS = 8;      // rows per step of a workgroup, read four at a time
constexpr int MV2_HALF = 4;

// The b words of this lane's 32 columns for four consecutive rows (rows past r repeat the last one).  n is a multiple
// of 32 here, so a lane's words are all inside the row or all outside; `w0` is clamped by the caller for the latter,
// whose vector entries are zero.
template <int BITS>
__device__ __forceinline__ void mv_load_rows(uint32_t (&w)[MV2_HALF][BITS + 1], const PackedArgs& a, int rowbase, uint32_t w0) {
#pragma unroll
    for (int rr = 0; rr < MV2_HALF; ++rr) {
        // the row is the same for the whole wavefront: its address stays in scalar registers and the load takes the
        // lane's word offset as a 32-bit index (r and the words of a row fit 31 bits, checked on the host)
        const int row = __builtin_amdgcn_readfirstlane(min(rowbase + rr, (int)a.r - 1));
        const uint32_t* prow = a.words + (int64_t)row * a.ldp;
        struct __attribute__((packed, aligned(4))) Words { uint32_t v[BITS]; };
        const Words t = *reinterpret_cast<const Words*>(reinterpret_cast<const char*>(prow) + w0 * 4u);      // one load of b words
#pragma unroll
        for (int i = 0; i < BITS; ++i) w[rr][i] = t.v[i];
        w[rr][BITS] = 0u;
    }
}

// The same two instructions as volatile statements: they keep their program order, so a pair of halves is consumed by
// its dot product right after it is made.  Left to itself the scheduler makes all 64 pairs of four rows first and
// holds them in registers, which costs a wavefront per SIMD.
__device__ __forceinline__ uint32_t and_or_ordered(uint32_t a, uint32_t mask, uint32_t c) {
    uint32_t v;
    asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(v) : "v"(a), "s"(mask), "v"(c));
    return v;
}
__device__ __forceinline__ void dot2_ordered(float& d, uint32_t pair, half2v xv) {
    asm volatile("v_dot2_f32_f16 %0, %1, %2, %0" : "+v"(d) : "v"(pair), "v"(xv));
}

// acc[rr] += scale * (sum (2^b + code) x - (2^b + zero) sum x) over this lane's 32 columns, for four rows
template <int BITS>
__device__ __forceinline__ void mv_dot_rows(const uint32_t (&w)[MV2_HALF][BITS + 1], const half2v (&xq)[16], float sx, float* acc,
                                            const PackedArgs& a, int rowbase, uint32_t g0) {
    constexpr int WANT = 10 - BITS;
    constexpr uint32_t M = (1u << BITS) - 1u;
    constexpr uint32_t MASK_LO = M << WANT, MASK_HI = M << (16 + WANT), MASK = MASK_LO | MASK_HI;
    const uint32_t magic = 0x3C003C00u + (uint32_t)BITS * 0x04000400u;       // (2^b, 2^b) as two halves
    const float offset = (float)(1 << BITS);
#pragma unroll
    for (int rr = 0; rr < MV2_HALF; ++rr) {
        // two interleaved chains per row, so consecutive dot products do not wait for each other
        float d0 = 0.f, d1 = 0.f;
        uint32_t joined[3] = {0u, 0u, 0u};
        if constexpr (BITS == 3) {
            joined[0] = __builtin_amdgcn_perm(w[rr][1], w[rr][0], 0x07060100u);      // low half of w0, high half of w1
            joined[1] = __builtin_amdgcn_perm(w[rr][0], w[rr][2], 0x07060100u);      // low half of w2, high half of w0
            joined[2] = __builtin_amdgcn_perm(w[rr][2], w[rr][1], 0x07060100u);      // low half of w1, high half of w2
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const PairSpec sp = PairTable<BITS>::at(i);
            uint32_t v;
            if (sp.lo_word < 0) {
                const uint32_t ta = stream_bits<BITS>(w[rr], BITS * sp.k_lo - WANT);
                const uint32_t tb = stream_bits<BITS>(w[rr], BITS * sp.k_hi - (16 + WANT));
                v = and_or_ordered(tb, MASK_HI, and_or_ordered(ta, MASK_LO, magic));
            } else {
                uint32_t m;
                if (sp.lo_word == sp.hi_word) m = w[rr][sp.lo_word];
                else m = joined[sp.lo_word == 0 ? 0 : (sp.lo_word == 2 ? 1 : 2)];
                const uint32_t t = sp.rel >= WANT ? (m >> (sp.rel - WANT)) : (m << (WANT - sp.rel));
                v = and_or_ordered(t, MASK, magic);
            }
            if (i & 1) dot2_ordered(d1, v, xq[i]);
            else       dot2_ordered(d0, v, xq[i]);
        }
        const int row = __builtin_amdgcn_readfirstlane(min(rowbase + rr, (int)a.r - 1));
        const int64_t gbase = (int64_t)row * a.ngroups;      // scalar; the lane's group is a 32-bit index on top
        const float sc = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(a.scales + gbase) + g0 * 4u);
        const int zr = *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(a.zeros + gbase) + g0 * 4u);
        acc[rr] = fmaf(sc, (d0 + d1) - (offset + (float)zr) * sx, acc[rr]);
    }
}

// The words of the next four rows are requested before the current four are multiplied (within a segment, and across to
// the wavefront's next segment), so a wavefront always has loads in flight while it computes.
template <int BITS>
__global__ __launch_bounds__(256) void matvec_dot2_kernel(PackedArgs a, const __half* x, float* y) {
    __shared__ float part[4][MV2_ROWS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t nseg = (a.n + MV_SEG - 1) / MV_SEG;
    const int64_t row_end = min(((int64_t)blockIdx.x + 1) * a.rows_per_wg, a.r);
    for (int64_t row0 = (int64_t)blockIdx.x * a.rows_per_wg; row0 < row_end; row0 += MV2_ROWS) {
    float acc[MV2_ROWS];
#pragma unroll
    for (int rr = 0; rr < MV2_ROWS; ++rr) acc[rr] = 0.f;
    uint32_t wa[MV2_HALF][BITS + 1], wb[MV2_HALF][BITS + 1];
    const uint32_t wlast = (uint32_t)(a.words_per_row - BITS);      // n is a multiple of 32 and at least 32
    auto words_at = [&](int64_t seg) { return min((uint32_t)(((seg * MV_SEG) >> 5) + lane) * BITS, wlast); };
    const int row0i = (int)row0;
    if (wave < nseg) mv_load_rows<BITS>(wa, a, row0i, words_at(wave));
#pragma unroll 1
    for (int64_t s = wave; s < nseg; s += 4) {
        const int64_t k0 = s * MV_SEG + (int64_t)lane * 32;      // lanes past the last column: any words, zero vector entries
        mv_load_rows<BITS>(wb, a, row0i + MV2_HALF, words_at(s));
        uint32_t xp[16];                                     // the lane's 32 vector entries, two halves per register
        {
            const bool inside = k0 < a.n;
            const __half* xsrc = x + min(k0, a.n - 32);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 u = reinterpret_cast<const uint4*>(xsrc)[q];
                xp[4 * q] = inside ? u.x : 0u; xp[4 * q + 1] = inside ? u.y : 0u; xp[4 * q + 2] = inside ? u.z : 0u; xp[4 * q + 3] = inside ? u.w : 0u;
            }
        }
        asm volatile("" ::: "memory");                       // the requests above stay above the arithmetic below
        float sx = 0.f;
        half2v xq[16];                                       // the same entries paired like the codes
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, xp[i]), __builtin_bit_cast(half2v, 0x3C003C00u), sx, false);
            const PairSpec sp = PairTable<BITS>::at(i);
            const uint32_t lo = (xp[sp.k_lo >> 1] >> (16 * (sp.k_lo & 1))) & 0xFFFFu;
            const uint32_t hi = (sp.k_hi & 1) ? (xp[sp.k_hi >> 1] & 0xFFFF0000u) : (xp[sp.k_hi >> 1] << 16);
            xq[i] = __builtin_bit_cast(half2v, lo | hi);
        }
        // column / group size without the 64-bit division (n < 2^31 is checked on the host)
        const uint32_t kc = (uint32_t)min(k0, a.n - 32);
        const uint32_t g0 = a.group == 0 ? 0u : (a.gshift >= 0 ? kc >> a.gshift : kc / (uint32_t)a.group);
        mv_dot_rows<BITS>(wa, xq, sx, acc, a, row0i, g0);
        if (s + 4 < nseg) mv_load_rows<BITS>(wa, a, row0i, words_at(s + 4));
        asm volatile("" ::: "memory");
        mv_dot_rows<BITS>(wb, xq, sx, acc + MV2_HALF, a, row0i + MV2_HALF, g0);
    }
#pragma unroll
    for (int rr = 0; rr < MV2_ROWS; ++rr) {
        float v = acc[rr];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        if (lane == 0) part[wave][rr] = v;
    }
    __syncthreads();
    if (threadIdx.x < MV2_ROWS && row0 + threadIdx.x < a.r)
        y[row0 + threadIdx.x] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
    __syncthreads();
    }
}

// ---- one grid per row: the dot products on the matrix cores --------------------------------------------------------
// Same loads, same pairs of halves, but the pairs are not multiplied by v_dot2: two pair registers (4 weights) are the A
// operand and the two matching registers of the vector the B operand of one v_mfma_f32_16x16x16_f16.  The instruction
// computes D[i][j] += sum over the four lanes kb of <weights of lane (i, kb), vector entries of lane (j, kb)>
// (lane = i + 16 kb on the A side, j + 16 kb on the B side), so its DIAGONAL accumulates exactly the dot products the
// lanes want -- every lane's weights with its own vector entries, summed over four lanes at a time -- and the other 240
// entries (one lane's weights with another lane's entries) are never read.  That takes a third of the vector
// instructions off the path that bounds the kernel, at 8 matrix-core instructions per row and segment, which run beside
// the unpacking of other wavefronts.  With one grid per row the scale, the zero point and the 2^b offset come in at the
// very end:  y = scale (sum (2^b + code) x - (2^b + zero) sum x).
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));

// codes_as_half_pairs with the and-or written in C: what feeds a matrix-core instruction must be an instruction the
// compiler knows, so that it can keep the wait states the hardware wants between a vector write and the matrix read of
// the same register (an inline-assembly statement hides its instruction from that check).
template <int BITS>
__device__ __forceinline__ void codes_as_half_pairs_plain(const uint32_t (&w)[BITS + 1], uint32_t (&pr)[16]) {
    constexpr int WANT = 10 - BITS;
    constexpr uint32_t M = (1u << BITS) - 1u;
    constexpr uint32_t MASK_LO = M << WANT, MASK_HI = M << (16 + WANT), MASK = MASK_LO | MASK_HI;
    uint32_t magic = 0x3C003C00u + (uint32_t)BITS * 0x04000400u;             // (2^b, 2^b) as two halves
    // the constants in registers whose contents the compiler does not know: v_and_or_b32 takes no literals here, and with
    // known constants the compiler prefers an and and an or with one literal each
    uint32_t mask = MASK, mask_lo = MASK_LO, mask_hi = MASK_HI;
    asm volatile("" : "+s"(mask), "+s"(mask_lo), "+s"(mask_hi), "+v"(magic));
    uint32_t joined[3] = {0u, 0u, 0u};
    if constexpr (BITS == 3) {
        joined[0] = __builtin_amdgcn_perm(w[1], w[0], 0x07060100u);      // low half of w0, high half of w1
        joined[1] = __builtin_amdgcn_perm(w[0], w[2], 0x07060100u);      // low half of w2, high half of w0
        joined[2] = __builtin_amdgcn_perm(w[2], w[1], 0x07060100u);      // low half of w1, high half of w2
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const PairSpec sp = PairTable<BITS>::at(i);
        if (sp.lo_word < 0) {
            const uint32_t ta = stream_bits<BITS>(w, BITS * sp.k_lo - WANT);
            const uint32_t tb = stream_bits<BITS>(w, BITS * sp.k_hi - (16 + WANT));
            pr[i] = (tb & mask_hi) | ((ta & mask_lo) | magic);
        } else {
            uint32_t m;
            if (sp.lo_word == sp.hi_word) m = w[sp.lo_word];
            else m = joined[sp.lo_word == 0 ? 0 : (sp.lo_word == 2 ? 1 : 2)];
            const uint32_t t = sp.rel >= WANT ? (m >> (sp.rel - WANT)) : (m << (WANT - sp.rel));
            pr[i] = (t & mask) | magic;
        }
    }
}

template <int BITS>
__device__ __forceinline__ void mv_mfma_rows(const uint32_t (&w)[MV2_HALF][BITS + 1], const half2v (&xq)[16], float4v* acc) {
#pragma unroll
    for (int rr = 0; rr < MV2_HALF; ++rr) {
        uint32_t pr[16];
        codes_as_half_pairs_plain<BITS>(w[rr], pr);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const u32x2v av = {pr[2 * t], pr[2 * t + 1]};
            const u32x2v bv = {__builtin_bit_cast(uint32_t, xq[2 * t]), __builtin_bit_cast(uint32_t, xq[2 * t + 1])};
            acc[rr] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4v, av), __builtin_bit_cast(half4v, bv), acc[rr], 0, 0, 0);
        }
    }
}

template <int BITS>
__global__ __launch_bounds__(256) void matvec_mfma_kernel(PackedArgs a, const __half* x, float* y) {
    __shared__ float part[4][MV2_ROWS + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t nseg = (a.n + MV_SEG - 1) / MV_SEG;
    const int64_t row_end = min(((int64_t)blockIdx.x + 1) * a.rows_per_wg, a.r);
    // this lane's element of the diagonal of D: lane = j + 16 ib holds D[4 ib + e][j], e = 0 .. 3
    const int dj = lane & 15, dib = lane >> 4;
    const bool on_diag = (dj >> 2) == dib;
    const int de = dj & 3;
    for (int64_t row0 = (int64_t)blockIdx.x * a.rows_per_wg; row0 < row_end; row0 += MV2_ROWS) {
    float4v acc[MV2_ROWS];
#pragma unroll
    for (int rr = 0; rr < MV2_ROWS; ++rr) acc[rr] = float4v{0.f, 0.f, 0.f, 0.f};
    float sx = 0.f;                                          // sum of this lane's vector entries over its segments
    uint32_t wa[MV2_HALF][BITS + 1], wb[MV2_HALF][BITS + 1];
    const uint32_t wlast = (uint32_t)(a.words_per_row - BITS);      // n is a multiple of 32 and at least 32
    auto words_at = [&](int64_t seg) { return min((uint32_t)(((seg * MV_SEG) >> 5) + lane) * BITS, wlast); };
    const int row0i = (int)row0;
    if (wave < nseg) mv_load_rows<BITS>(wa, a, row0i, words_at(wave));
#pragma unroll 1
    for (int64_t s = wave; s < nseg; s += 4) {
        const int64_t k0 = s * MV_SEG + (int64_t)lane * 32;      // lanes past the last column: any words, zero vector entries
        mv_load_rows<BITS>(wb, a, row0i + MV2_HALF, words_at(s));
        uint32_t xp[16];
        {
            const bool inside = k0 < a.n;
            const __half* xsrc = x + min(k0, a.n - 32);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint4 u = reinterpret_cast<const uint4*>(xsrc)[q];
                xp[4 * q] = inside ? u.x : 0u; xp[4 * q + 1] = inside ? u.y : 0u; xp[4 * q + 2] = inside ? u.z : 0u; xp[4 * q + 3] = inside ? u.w : 0u;
            }
        }
        asm volatile("" ::: "memory");                       // the requests above stay above the arithmetic below
        half2v xq[16];                                       // the same entries paired like the codes
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, xp[i]), __builtin_bit_cast(half2v, 0x3C003C00u), sx, false);
            const PairSpec sp = PairTable<BITS>::at(i);
            const uint32_t lo = (xp[sp.k_lo >> 1] >> (16 * (sp.k_lo & 1))) & 0xFFFFu;
            const uint32_t hi = (sp.k_hi & 1) ? (xp[sp.k_hi >> 1] & 0xFFFF0000u) : (xp[sp.k_hi >> 1] << 16);
            xq[i] = __builtin_bit_cast(half2v, lo | hi);
        }
        mv_mfma_rows<BITS>(wa, xq, acc);
        if (s + 4 < nseg) mv_load_rows<BITS>(wa, a, row0i, words_at(s + 4));
        asm volatile("" ::: "memory");
        mv_mfma_rows<BITS>(wb, xq, acc + MV2_HALF);
    }
#pragma unroll
    for (int rr = 0; rr <= MV2_ROWS; ++rr) {
        float v;
        if (rr < MV2_ROWS) {
            const float4v c = acc[rr < MV2_ROWS ? rr : 0];
            const float e = de == 0 ? c.x : (de == 1 ? c.y : (de == 2 ? c.z : c.w));
            v = on_diag ? e : 0.f;
        } else {
            v = sx;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        if (lane == 0) part[wave][rr] = v;
    }
    __syncthreads();
    if (threadIdx.x < MV2_ROWS && row0 + threadIdx.x < a.r) {
        const int64_t row = row0 + threadIdx.x;
        const float dots = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
        const float sxs = (part[0][MV2_ROWS] + part[1][MV2_ROWS]) + (part[2][MV2_ROWS] + part[3][MV2_ROWS]);
        y[row] = a.scales[row * a.ngroups] * (dots - ((float)(1 << BITS) + (float)a.zeros[row * a.ngroups]) * sxs);
    }
    __syncthreads();
    }
}

__global__ void zero_vector_kernel(float* y, int64_t r) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < r) y[i] = 0.f;
}

static int check_packed(const char* who, const uint32_t* words, int64_t ldp, int64_t r, int64_t n, int bits,
                        const float* scales, const int32_t* zeros, int64_t group, PackedArgs* a) {
    if (r < 0 || n < 0) return fail(GPTQ_ERR_INVALID_ARG, "%s: negative size", who);
    if (bits < 2 || bits > 4) return fail(GPTQ_ERR_INVALID_ARG, "%s: bits must be 2, 3 or 4 (got %d)", who, bits);
    if (group < 0) return fail(GPTQ_ERR_INVALID_ARG, "%s: negative group", who);
    if (group > 0 && n % group) return fail(GPTQ_ERR_INVALID_ARG, "%s: n must be a multiple of the group size", who);
    if (r == 0 || n == 0) return GPTQ_OK;
    if (!words || !scales || !zeros) return fail(GPTQ_ERR_INVALID_ARG, "%s: null pointer", who);
    const int64_t wpr = (n * bits + 31) / 32;
    if (ldp < wpr) return fail(GPTQ_ERR_INVALID_ARG, "%s: word pitch smaller than ceil(n*bits/32)", who);
    a->words = words; a->ldp = ldp; a->r = r; a->n = n; a->words_per_row = wpr;
    a->scales = scales; a->zeros = zeros; a->group = group; a->ngroups = group ? n / group : 1;
    a->gshift = -1;
    if (group > 0 && (group & (group - 1)) == 0) { int sh = 0; while (((int64_t)1 << sh) < group) ++sh; a->gshift = sh; }
    return -1;
}

}  // namespace gptq

using namespace gptq;

extern "C" int gptq_dequantize_packed(const uint32_t* words, int64_t ldp, int64_t r, int64_t n, int bits,
                                      const float* scales, const int32_t* zeros, int64_t group,
                                      void* out, int odtype, int64_t ldo, void* stream) {
    PackedArgs a{};
    const int rc = check_packed("dequantize_packed", words, ldp, r, n, bits, scales, zeros, group, &a);
    if (rc >= 0) return rc;
    if (odtype != GPTQ_F16 && odtype != GPTQ_F32) return fail(GPTQ_ERR_INVALID_ARG, "dequantize_packed: output type must be float16 or float32");
    if (!out) return fail(GPTQ_ERR_INVALID_ARG, "dequantize_packed: null pointer");
    if (ldo < n) return fail(GPTQ_ERR_INVALID_ARG, "dequantize_packed: ldo < n");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t osz = odtype == GPTQ_F16 ? 2 : 4;
    if (n % 8 == 0 && n < 0x7fffffffLL && (group == 0 || group % 8 == 0) && aligned(out, 16) && (ldo * osz) % 16 == 0) {
        const int64_t octets = n / 8;
        const dim3 grid((unsigned)std::min<int64_t>(r, 256 * 64));
#define GPTQ_DQ8(B)                                                                                                              \
        if (odtype == GPTQ_F16) hipLaunchKernelGGL((dequantize8_kernel<B, _Float16>), grid, dim3(256), 0, s, a, static_cast<_Float16*>(out), ldo, octets); \
        else hipLaunchKernelGGL((dequantize8_kernel<B, float>), grid, dim3(256), 0, s, a, static_cast<float*>(out), ldo, octets)
        if (bits == 2) { GPTQ_DQ8(2); } else if (bits == 3) { GPTQ_DQ8(3); } else { GPTQ_DQ8(4); }
#undef GPTQ_DQ8
        GPTQ_LAUNCH_CHECK();
        return GPTQ_OK;
    }
    const int64_t g32 = (n + 7) / 8;               // octets of codes per row
    if (r * g32 > (int64_t)0x7fffffff * 256) return fail(GPTQ_ERR_UNSUPPORTED, "dequantize_packed: too large");
    const unsigned blocks = (unsigned)ceil_div(r * g32, 256);
#define GPTQ_DQ(B)                                                                                                              \
    if (odtype == GPTQ_F16) hipLaunchKernelGGL((dequantize_kernel<B, __half>), dim3(blocks), dim3(256), 0, s, a, static_cast<__half*>(out), ldo, g32); \
    else hipLaunchKernelGGL((dequantize_kernel<B, float>), dim3(blocks), dim3(256), 0, s, a, static_cast<float*>(out), ldo, g32)
    if (bits == 2) { GPTQ_DQ(2); } else if (bits == 3) { GPTQ_DQ(3); } else { GPTQ_DQ(4); }
#undef GPTQ_DQ
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}

// Rows are dealt to about eight workgroups per CU (what the kernels' registers allow) in equal shares, each a
// multiple of the kernel's row chunk: with one chunk per workgroup the last round of a large launch would run
// the chip partly empty.
static int64_t rows_per_workgroup(int64_t r, int chunk) {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
        else cus = 256;
    }
    const int64_t slots = (int64_t)cus * 8;
    return (int64_t)round_up((size_t)ceil_div(r, slots), (size_t)chunk);
}

template <int BITS, typename XT>
static void launch_matvec(PackedArgs a, const XT* x, float* y, hipStream_t s) {
    const int gsub = (a.group == 0 || a.group % 32 == 0) ? 1 : (int)(32 / a.group);
    if constexpr (sizeof(XT) == 2) {
        // the fast kernel wants whole lanes (32 columns each) and 16-byte loads of the vector
        if (gsub == 1 && a.n % 32 == 0 && a.n >= 32 && a.n < 0x7fffffffLL && a.r < 0x7fffffffLL && a.words_per_row < 0x3fffffffLL &&
            a.ngroups < 0x3fffffffLL && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
            a.rows_per_wg = rows_per_workgroup(a.r, MV2_ROWS);
            if (a.group == 0)
                hipLaunchKernelGGL((matvec_mfma_kernel<BITS>), dim3((unsigned)ceil_div(a.r, a.rows_per_wg)), dim3(256), 0, s, a, x, y);
            else
                hipLaunchKernelGGL((matvec_dot2_kernel<BITS>), dim3((unsigned)ceil_div(a.r, a.rows_per_wg)), dim3(256), 0, s, a, x, y);
            return;
        }
    }
    a.rows_per_wg = rows_per_workgroup(a.r, MV_ROWS);
    const unsigned blocks = (unsigned)ceil_div(a.r, a.rows_per_wg);
    if (gsub == 1) hipLaunchKernelGGL((matvec_kernel<BITS, 1, XT>), dim3(blocks), dim3(256), 0, s, a, x, y);
    else if (gsub == 2) hipLaunchKernelGGL((matvec_kernel<BITS, 2, XT>), dim3(blocks), dim3(256), 0, s, a, x, y);
    else hipLaunchKernelGGL((matvec_kernel<BITS, 4, XT>), dim3(blocks), dim3(256), 0, s, a, x, y);
}

extern "C" int gptq_matvec_packed(const uint32_t* words, int64_t ldp, int64_t r, int64_t n, int bits,
                                  const float* scales, const int32_t* zeros, int64_t group,
                                  const void* x, int xdtype, float* y, void* stream) {
    PackedArgs a{};
    const int rc = check_packed("matvec_packed", words, ldp, r, n, bits, scales, zeros, group, &a);
    if (rc >= 0) {
        if (rc == GPTQ_OK && r > 0 && n == 0) {          // an empty sum: y = 0
            if (!y) return fail(GPTQ_ERR_INVALID_ARG, "matvec_packed: null pointer");
            hipLaunchKernelGGL(zero_vector_kernel, dim3((unsigned)ceil_div(r, 256)), dim3(256), 0, static_cast<hipStream_t>(stream), y, r);
            GPTQ_LAUNCH_CHECK();
        }
        return rc;
    }
    if (xdtype != GPTQ_F16 && xdtype != GPTQ_F32) return fail(GPTQ_ERR_INVALID_ARG, "matvec_packed: vector type must be float16 or float32");
    if (!x || !y) return fail(GPTQ_ERR_INVALID_ARG, "matvec_packed: null pointer");
    if (group > 0 && group % 32 && group != 8 && group != 16)
        return fail(GPTQ_ERR_UNSUPPORTED, "matvec_packed: group size %lld not built (8, 16 or a multiple of 32)", (long long)group);
    if (ceil_div(r, MV_ROWS) > 0x7fffffffLL) return fail(GPTQ_ERR_UNSUPPORTED, "matvec_packed: too many rows");
    hipStream_t s = static_cast<hipStream_t>(stream);
#define GPTQ_MV(B)                                                                              \
    if (xdtype == GPTQ_F16) launch_matvec<B, __half>(a, static_cast<const __half*>(x), y, s);   \
    else launch_matvec<B, float>(a, static_cast<const float*>(x), y, s)
    if (bits == 2) { GPTQ_MV(2); } else if (bits == 3) { GPTQ_MV(3); } else { GPTQ_MV(4); }
#undef GPTQ_MV
    GPTQ_LAUNCH_CHECK();
    return GPTQ_OK;
}
