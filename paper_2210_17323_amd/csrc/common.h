// Shared host-side helpers of the GPTQ gfx950 library: status codes, error text, launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <initializer_list>
#include <cstdint>
#include <cstdio>

#include "../../include/gptq.h"

namespace gptq {

void set_error(const char* fmt, ...);

inline int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int fail_v(int code, const char* fmt, va_list ap);
inline int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    int rc = fail_v(code, fmt, ap);
    va_end(ap);
    return rc;
}

#define GPTQ_HIP_CHECK(expr)                                                                      \
    do {                                                                                          \
        hipError_t _e = (expr);                                                                   \
        if (_e != hipSuccess)                                                                     \
            return ::gptq::fail(GPTQ_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e));     \
    } while (0)

#define GPTQ_LAUNCH_CHECK() GPTQ_HIP_CHECK(hipGetLastError())

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t round_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- look-ahead: a helper stream and a ring of events (runtime.hip) ----------------------------
// The blocked solvers put the short, serial kernels of the next block column and the long trailing GEMM
// of the current one on two streams so that they overlap.  The helper stream (default priority,
// non-blocking) and its events are created once per host thread and device and live until the process
// ends.  Every use forks from and joins back into the caller's stream with events, so after an entry
// point returns all of its work is ordered on the caller's stream alone.
struct Lookahead {
    hipStream_t stream = nullptr;       // long trailing updates
    hipStream_t stream2 = nullptr;      // the short kernels that trail the factorisation's serial chain: the next block's strip
    hipStream_t stream3 = nullptr;      // ... and the inverse of the diagonal block
    hipEvent_t ev[32] = {};
    unsigned next = 0;
    hipEvent_t event() { return ev[next++ & 31]; }
};
int lookahead_get(Lookahead** out);     // for the current device; GPTQ_OK or an error code

// The streams of one entry point.  open(s, true) forks onto the library's helper streams; open(s, false) keeps
// everything on the caller's stream (every side stream == main, no events: the same kernels in an order that respects
// every dependence, without overlap) -- for callers that must not create streams or events.  The destructor joins
// the helper streams back into the caller's on EVERY return path, so also after a launch failed half way through a
// call nothing is left running unordered beside the caller's stream.  An event of the ring may be recorded again
// while an earlier wait on it is still pending: a wait refers to the record that was current when it was enqueued.
struct TwoStreams {
    hipStream_t main = nullptr, side = nullptr, side2 = nullptr, side3 = nullptr;
    Lookahead* la = nullptr;
    int open(hipStream_t s, bool lookahead) {
        main = side = side2 = side3 = s;
        if (!lookahead) return GPTQ_OK;
        if (int rc = lookahead_get(&la)) return rc;
        side = la->stream;
        side2 = la->stream2;
        side3 = la->stream3;
        // fork: nothing on a helper stream may start before the work already on the caller's stream (a helper's first
        // kernel may touch memory -- a workspace, say -- that earlier work of the caller still writes)
        hipEvent_t fork = la->event();
        GPTQ_HIP_CHECK(hipEventRecord(fork, main));
        for (hipStream_t st : {side, side2, side3}) GPTQ_HIP_CHECK(hipStreamWaitEvent(st, fork, 0));
        return GPTQ_OK;
    }
    // *ev = a point on `on` that wait() can order another stream behind; stays null in single-stream mode
    int mark(hipStream_t on, hipEvent_t* ev) {
        *ev = nullptr;
        if (!la) return GPTQ_OK;
        hipEvent_t e = la->event();
        GPTQ_HIP_CHECK(hipEventRecord(e, on));
        *ev = e;
        return GPTQ_OK;
    }
    int wait(hipStream_t who, hipEvent_t ev) {
        if (!la || !ev) return GPTQ_OK;
        GPTQ_HIP_CHECK(hipStreamWaitEvent(who, ev, 0));
        return GPTQ_OK;
    }
    ~TwoStreams() {
        if (!la) return;
        for (hipStream_t st : {side, side2, side3}) {
            hipEvent_t e = la->event();
            if (hipEventRecord(e, st) == hipSuccess) (void)hipStreamWaitEvent(main, e, 0);
        }
    }
};

// ---- float32 matrix-core GEMM used by several steps (gemm_f32.hip) --------------------------
// C[M x N] += alpha * A[M x K] * op(B), A row-major (K contiguous).
//   b_is_nk = true : B is [N x K] row-major (K contiguous)  -> C += alpha * A * B^T
//   b_is_nk = false: B is [K x N] row-major (N contiguous)  -> C += alpha * A * B
//   overwrite: C = alpha * A * op(B) instead of accumulating.
//   upper_only: skip 128x128 output tiles that lie entirely below the diagonal (row0 > col0 + 127),
//               with (crow0, ccol0) the global offset of C's first element inside its parent matrix.
//   a_upper_tri: A[M x K] is the top-left part of an upper-triangular matrix (A[i][k] == 0 for k < i
//               rounded down to 128): the K loop of a tile starts at the tile's first row.
//   b_upper_tri: B given as [K x N] is the top-left part of an upper-triangular matrix with explicit zeros
//               below the diagonal: the K loop of a tile may end at the tile's last column (the large-tile
//               kernels do that; where it is not done the zeros give the same result).
// All pointers 16-byte aligned, leading dimensions multiples of 4.
struct GemmF32 {
    const float* A; int64_t lda;
    const float* B; int64_t ldb;
    float* C; int64_t ldc;
    int64_t M, N, K;
    float alpha;
    bool b_is_nk;
    bool overwrite;
    bool upper_only;
    int64_t crow0, ccol0;
    bool a_upper_tri;   // A is upper triangular with zeros below its diagonal blocks: skip k < first row of the tile
    bool b_upper_tri;   // B [K x N] is upper triangular with zeros below the diagonal: skip k > last column of the tile
    int max_workgroups; // > 0: a launch of large tiles uses at most this many workgroups (each walks several tiles), which
                        //      leaves the other CUs to kernels of other streams; workgroup w runs on XCD w % 8, so a
                        //      multiple of 8 below the CU count frees the same number of CUs on every XCD
};
int launch_gemm_f32(const GemmF32& g, hipStream_t s);

// ---- float32 products of rank 1024 on the bf16 matrix cores (gemm_split.hip) -----------------
// C[256 tiles_m x 256 tiles_n] += alpha * A * B^T over K = SPLIT_K, with both operands given as "planes": the three
// bfloat16 pieces of every float32 element in the blocked layout the kernel copies straight into LDS.
//   launch_split_rows: A [rows x SPLIT_K] float32, K contiguous        -> planes of ceil(rows / 256) panels
//   launch_split_cols: B [SPLIT_K x cols] float32, columns contiguous  -> planes of ceil(cols / 256) panels (of B^T)
// Both write split_planes_bytes(rows) bytes, the last 16 KB of which are zeros (split_zero_block); rows past the
// operand's end are zeros.  A launch reads panels a_panel0 .. and b_panel0 .. of the two plane buffers.
//   upper_square: C is square and only the tiles of its upper triangle are computed (diagonal tiles whole).
//   skip_lower:   rectangular C at (crow0, ccol0) of a parent matrix: tiles entirely below the parent's diagonal are left out.
// The six piece products kept leave a relative error of at most 2^-23 per product of two elements.
constexpr int SPLIT_K = 1024;
struct SplitGemm {
    const unsigned char* A_planes; int a_panel0;
    const unsigned char* B_planes; int b_panel0;
    const unsigned char* A_zero;        // each operand's block of zeros: split_zero_block(planes, rows given to its split)
    const unsigned char* B_zero;
    float* C; int64_t ldc;
    float alpha;
    int tiles_m, tiles_n;
    bool upper_square;
    bool skip_lower; int64_t crow0, ccol0;
};
size_t split_planes_bytes(int64_t rows);
bool split_pays(int64_t tiles);         // whether a launch of that many 256 x 256 tiles should take the split kernel
inline const unsigned char* split_zero_block(const unsigned char* planes, int64_t rows) { return planes + split_planes_bytes(rows) - 16384; }
int launch_split_rows(const float* A, int64_t lda, int64_t rows, unsigned char* planes, hipStream_t s);
int launch_split_cols(const float* B, int64_t ldb, int64_t cols, unsigned char* planes, hipStream_t s);
int launch_gemm_split(const SplitGemm& g, hipStream_t s);

}  // namespace gptq
