/*
 * gptq.h -- C ABI of the MI355X (gfx950) GPTQ per-layer quantization solver.
 *
 * The calls follow the steps of the GPTQ algorithm (Frantar et al., arXiv 2210.17323):
 *   1. gptq_hessian_accumulate      H += 2 X X^T over chunks of calibration tokens  (Section 2; Alg. 1 caption)
 *   2. gptq_damp_cholesky_inverse   U = Cholesky((H + lambda I)^-1)^T                (Section 3, Step 3; Alg. 1)
 *   3. gptq_quantize_layer          the block / column loop with lazy batch updates  (Section 3, Step 2; Alg. 1)
 *   4. gptq_pack                    dense 2/3/4-bit stream of the resulting codes    (Section 4, "Practical Speedups")
 * and two consumers of the packed layer (same section): gptq_dequantize_packed, gptq_matvec_packed.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer to memory owned by the caller, valid on the current
 *     HIP device; the library never allocates or frees device memory.  Scratch space comes from a
 *     caller-provided workspace whose size the matching *_workspace_bytes call returns (one variant,
 *     gptq_damp_cholesky_inverse_noalloc, uses a fixed array that is part of the library instead).
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues work on that stream and returns; it never synchronises.
 *   - Return value: GPTQ_OK or an error code; gptq_last_error() (thread-local) describes the problem.
 *     Arguments are validated on the host before any launch: GPTQ_ERR_INVALID_ARG, GPTQ_ERR_UNSUPPORTED and
 *     GPTQ_ERR_WORKSPACE mean that nothing has been enqueued.  GPTQ_ERR_HIP (a launch or runtime call failed
 *     part way through) may leave earlier kernels of the call enqueued: the outputs are then undefined, but
 *     all of that work is ordered on `stream` (the library's helper stream is joined back on every return
 *     path), so synchronising `stream` is enough before the buffers are reused or freed.  No C++ exception
 *     crosses this boundary.
 *   - Not re-entrant on the same workspace: two calls sharing a workspace must be on the same stream.
 */
#ifndef GPTQ_MI355_H
#define GPTQ_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GPTQ_API __attribute__((visibility("default")))

enum {
    GPTQ_OK = 0,
    GPTQ_ERR_INVALID_ARG = 1,      /* null pointer, bad size, bad alignment, bad enum                   */
    GPTQ_ERR_NOT_POSDEF = 2,       /* reported by gptq_check_info when a pivot was not positive          */
    GPTQ_ERR_HIP = 3,              /* a HIP runtime call failed                                          */
    GPTQ_ERR_UNSUPPORTED = 4,      /* valid request this build has no kernel for                         */
    GPTQ_ERR_WORKSPACE = 5         /* workspace pointer null or smaller than *_workspace_bytes            */
};

enum { GPTQ_F16 = 0, GPTQ_BF16 = 1, GPTQ_F32 = 2 };          /* element types of X and W              */
enum { GPTQ_GRID_MINMAX = 0, GPTQ_GRID_TERNARY = 1 };        /* quantization grids                    */

GPTQ_API int gptq_version(void);
GPTQ_API const char* gptq_last_error(void);

/*
 * The only state the library keeps between calls: three helper streams (default priority, non-blocking) and 32 events per
 * host thread and device, created by the first call of gptq_damp_cholesky* / gptq_quantize_layer* on that thread and
 * device and used by the later ones (two caller streams of one thread therefore share them: their calls are correct
 * but do not overlap each other's helper work).  gptq_release_thread_resources waits for the calling thread's helper
 * streams on the current device and destroys them and their events; the next call that needs them creates new ones.
 * It must not be called while a HIP graph capture that includes a library call is in progress on this thread, and
 * graphs captured earlier stay valid (a graph does not refer to the streams it was captured on).  GPTQ_OK also when
 * there was nothing to release.
 */
GPTQ_API int gptq_release_thread_resources(void);

/*
 * Step 1 -- Hessian of the layer-wise objective, H = 2 X X^T (Section 2, text before Eq. 2; Alg. 1 caption).
 *
 *   H   [n x n] float32, ldh >= n.  Accumulated in place: H += 2 X X^T.  The caller zero-fills H
 *       before the first chunk.  Only the UPPER triangle (column >= row) is defined afterwards;
 *       entries below the diagonal hold unspecified partial values until gptq_hessian_symmetrize.
 *   X   [n x t] one row per input channel, t tokens contiguous (ldx >= t), type xdtype
 *       (GPTQ_F16 / GPTQ_BF16: products are exact in float32 and accumulated in float32 by the
 *       matrix cores; GPTQ_F32: float32 matrix-core products).
 *       X must be 16-byte aligned and ldx a multiple of 8 (f16/bf16) or 4 (f32) elements.
 *   ws  optional workspace (may be NULL) of gptq_hessian_accumulate_workspace_bytes(n, t, xdtype) bytes,
 *       256-byte aligned.  With it, 16-bit chunks of layers with at least 2048 channels are first repacked
 *       so that every 256-channel x 32-token panel step is one contiguous 16 KB block, which the
 *       matrix-core kernel copies with far better cache-line and DRAM-page locality; for layers whose H has
 *       few 256 x 256 tiles (up to ~16000 channels) the token range of the call is also split in up to 8
 *       parts whose partial tiles (held in the workspace) are added in a fixed order, so that all CUs have
 *       work -- pass such layers long chunks, whole calibration sets if they fit.  Without the workspace
 *       the kernels read X in place: the same sums up to float32 summation order, at lower speed.
 *       Calls of more than 32768 tokens on layers whose H fills the chip without that split (from ~11000 channels
 *       on) walk the token range in slices of 32768: the workspace then holds two repacked slices, and every slice
 *       but the first is repacked inside the preceding slice's matrix-core kernel by the workgroups that have run
 *       out of tiles, so the repack costs no pass of its own -- pass such layers whole calibration sets too.
 *       gptq_hessian_accumulate_launches(n, t, xdtype) tells how many launches of the matrix-core kernel a call
 *       makes (1 unless it is sliced).  The environment variable GPTQ_HESSIAN_SLICE_TOKENS (a multiple of 32), read
 *       at every call, changes the slice length and makes every 16-bit call longer than a slice take this path.
 *       Repeating a call gives the same bits either way.  The size is 0 where the workspace is not used (ws is
 *       then ignored).  A non-NULL ws that is misaligned or smaller than that size is GPTQ_ERR_WORKSPACE.
 *   No normalisation by the token count is applied (the quantization result is invariant to the
 *   scale of H).  n == 0 or t == 0 is a valid no-op.
 */
GPTQ_API size_t gptq_hessian_accumulate_workspace_bytes(int64_t n, int64_t t, int xdtype);
GPTQ_API int64_t gptq_hessian_accumulate_launches(int64_t n, int64_t t, int xdtype);
GPTQ_API int gptq_hessian_accumulate(float* H, int64_t ldh, const void* X, int xdtype,
                            int64_t n, int64_t t, int64_t ldx, void* ws, size_t ws_bytes, void* stream);

/*
 * Step 1 for token-major activations: X is [t x n] (one row per token, channels contiguous, ldx >= n) -- the
 * layout of a layer's input in a framework -- of type float16 or bfloat16; H[upper] += 2 X^T X.  Same arithmetic
 * and result as gptq_hessian_accumulate on the transposed chunk with its workspace.  The workspace is required:
 * gptq_hessian_accumulate_token_major_workspace_bytes(n, t, xdtype) bytes, 256-byte aligned.  X 16-byte
 * aligned, ldx % 8 == 0.  float32 activations are not taken in this layout (GPTQ_ERR_UNSUPPORTED).
 */
GPTQ_API size_t gptq_hessian_accumulate_token_major_workspace_bytes(int64_t n, int64_t t, int xdtype);
GPTQ_API int gptq_hessian_accumulate_token_major(float* H, int64_t ldh, const void* X, int xdtype,
                                        int64_t n, int64_t t, int64_t ldx, void* ws, size_t ws_bytes, void* stream);

/* Copies the upper triangle of H onto the lower one (H[j][i] = H[i][j] for j > i). */
GPTQ_API int gptq_hessian_symmetrize(float* H, int64_t ldh, int64_t n, void* stream);

/*
 * Step 2 -- dampening and the Cholesky factor of the inverse (Section 3, Step 3; Alg. 1, third statement).
 *
 *   lambda = percdamp * mean(diag H)  ("1% of the average diagonal value": percdamp = 0.01);
 *   U = Cholesky((H + lambda I)^-1)^T, upper triangular with positive diagonal and
 *   (H + lambda I)^-1 = U^T U.  Row j of U from the diagonal on is what Alg. 1 reads.
 *
 *   H_U       [n x n] float32, ld >= n.  In: only the upper triangle of H is read.  Out: U in the
 *             upper triangle, zeros strictly below the diagonal.
 *   ws        workspace of at least gptq_damp_cholesky_inverse_workspace_bytes(n) bytes, 256-byte aligned.
 *   info_dev  device int.  Set to 0, or to the 1-based index of a column whose pivot was not
 *             positive (then U is meaningless).  Read it after synchronising, e.g. through
 *             gptq_check_info.  percdamp < 0 is invalid; percdamp == 0 is allowed.
 *   Computed as a Cholesky factorisation taken from the last column backwards, H + lambda I = R R^T with R
 *   upper triangular, followed by the triangular inverse U = R^-1 (the same matrix, by uniqueness of
 *   the Cholesky factor), all in float32; the rank-1024 updates that carry most of the flops multiply three-piece
 *   bfloat16 splits of their float32 operands on the bf16 matrix cores when they are large (see
 *   gptq_symmetric_update_split below: the error of a float32 multiply-add), which is also what the second half of
 *   the workspace is for.
 *   Part of the work is enqueued on helper streams owned by the library (created once per host thread and
 *   device, default priority) and joined back with events: when the call returns, everything it enqueued
 *   is ordered on `stream`, and nothing of it starts before the work already on `stream`.
 */
GPTQ_API size_t gptq_damp_cholesky_inverse_workspace_bytes(int64_t n);
GPTQ_API int gptq_damp_cholesky_inverse(float* H_U, int64_t ld, int64_t n, float percdamp,
                               void* ws, size_t ws_bytes, int* info_dev, void* stream);

/*
 * Step 2 for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc) and therefore cannot bring a workspace: the same kernels and the same
 * result as gptq_damp_cholesky_inverse, with the scratch space in a fixed device array that is part of the
 * library image (float32 kernels only; about 51 MiB, resident on every GPU the library runs on until the process ends).
 *
 *   n <= GPTQ_NOALLOC_MAX_N (gptq_noalloc_max_n() returns it); a larger n is GPTQ_ERR_UNSUPPORTED and nothing is
 *   enqueued.  H_U, ld, percdamp, info_dev and the result are as for gptq_damp_cholesky_inverse.
 *   The call allocates nothing and creates no stream or event: all kernels are enqueued on `stream` alone (no
 *   helper stream).  The first call on a device looks the array's address up once (hipGetSymbolAddress); make
 *   that call outside a graph capture.
 *   All calls on one GPU share that GPU's array: two such calls that overlap in time on one GPU (different
 *   streams, different threads) race and give undefined results -- order them.  Nothing in the array has to
 *   survive between calls and nothing has to be cleared: every region is written before it is read.
 */
#define GPTQ_NOALLOC_MAX_N 4096
GPTQ_API int64_t gptq_noalloc_max_n(void);
GPTQ_API int gptq_damp_cholesky_inverse_noalloc(float* H_U, int64_t ld, int64_t n, float percdamp,
                                       int* info_dev, void* stream);

/* Synchronises `stream`, reads *info_dev and returns GPTQ_OK or GPTQ_ERR_NOT_POSDEF
 * (the failing 1-based column index is stored in *host_info if host_info is not NULL). */
GPTQ_API int gptq_check_info(const int* info_dev, int* host_info, void* stream);

/*
 * Step 3 -- Algorithm 1: quantize W column by column in lazy blocks with error propagation.
 *
 *   W        [r x n] weights (rows = output features), type wdtype, ldw >= n.  Not modified: the
 *            solver works on a float32 copy held in the workspace.
 *   U        [n x n] float32 upper triangular factor from step 2, ldu >= n.
 *   bits     2, 3 or 4 for GPTQ_GRID_MINMAX (codes in [0, 2^bits - 1]); ignored for
 *            GPTQ_GRID_TERNARY (codes {0,1,2} = {-s, 0, +s}, zero point 1).
 *   grid     GPTQ_GRID_MINMAX: uniform asymmetric min-max grid (Section 4, Setup), range widened to
 *            contain 0: scale = (max(w,0) - min(w,0)) / maxq, zero = rint(-min(w,0)/scale), all-zero
 *            input: scale 1, zero 0.  GPTQ_GRID_TERNARY: s = max|w| (1 if all zero).
 *            code = clamp(rint(w/scale) + zero, 0, maxq), ties to even, evaluated in float32.
 *   block    lazy-batch block size B (Section 3, Step 2).  This build supports B = 128.
 *   group    0: one grid per row, fixed from the original W before the process.  g > 0: a new grid
 *            for columns [j, j+g) whenever j % g == 0, taken from the current updated weights
 *            (Section 4, "175 Billion Parameter Models").  Requires n % g == 0 and either
 *            128 % g == 0 with g >= 8, or g % 128 == 0.
 *   codes    [r x n] uint8 out, ldc >= n.
 *   scales   [r x G] float32 out, zeros [r x G] int32 out, G = 1 (group == 0) or n / group; dense.
 *   Wq       optional [r x n] float32 out (ldq >= n): the dequantised weights scale*(code - zero); may be NULL.
 *   half_E2_rows  optional [r] float64 out: per row, (1/2) * sum over columns of E^2 where
 *            E[:, j] = (W[:, j] - Q[:, j]) / U[j][j] at the time column j is quantized (Alg. 1).  Its
 *            sum over rows equals (1/2) tr((W-Q)(H + lambda I)(W-Q)^T).  May be NULL.
 *   ws       at least gptq_quantize_layer_workspace_bytes(r, n, block, group) bytes, 256-byte aligned.
 *   The update of column j's block and the rank-128 updates inside an outer block of 1024 columns are float32; the
 *   deferred rank-1024 updates beyond it are float32 matrix-core products or, when large, the split products of
 *   gptq_trailing_update_split below.
 *   r == 0 or n == 0 is a valid no-op.  Like step 2, the call puts part of its work on the library's helper
 *   stream and joins it back before returning.
 */
GPTQ_API size_t gptq_quantize_layer_workspace_bytes(int64_t r, int64_t n, int block, int64_t group);
GPTQ_API int gptq_quantize_layer(const void* W, int wdtype, int64_t ldw, int64_t r, int64_t n,
                        const float* U, int64_t ldu,
                        int bits, int grid, int block, int64_t group,
                        uint8_t* codes, int64_t ldc, float* scales, int32_t* zeros,
                        float* Wq, int64_t ldq, double* half_E2_rows,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Steps 2 and 3 without the inverse.  Alg. 1 can be driven by R, the Cholesky factor of H + lambda I itself
 * (H + lambda I = R R^T, R upper triangular), instead of U = Cholesky((H + lambda I)^-1)^T = R^-1: with
 * d_i = w_i - q_i (original weight minus its grid value) for the columns already quantized, the weight Alg. 1 holds
 * at column j is w_j + (sum_{i<j} d_i R[i][j]) / R[j][j] (the minimiser of Eq. 1 over the free columns makes
 * (delta R)_k vanish there), and its scaled error is e_j = (that weight - q_j) R[j][j] because U[j][j] = 1 / R[j][j]
 * (Section 3, Step 3; Eq. 2, Eq. 3).  Same codes as gptq_damp_cholesky_inverse + gptq_quantize_layer up to rounding
 * ties of the float32 arithmetic, at half the factorisation work (no triangular inverse).
 *
 * gptq_damp_cholesky: as gptq_damp_cholesky_inverse, but stops after the factorisation.  Out: R in the upper triangle
 *   of H_R, zeros strictly below.  Workspace and info_dev as there.
 * gptq_quantize_layer_from_factor: as gptq_quantize_layer with R in place of U.  group must be 0 (one grid per row)
 *   or 32, 64 or 128 (gptq_quantize_layer_from_factor_supports(group) returns 1 for these, 0 otherwise); any other
 *   group size is GPTQ_ERR_UNSUPPORTED here, use the U form.  A group's grid is taken from the weights as they stand at
 *   its first column (Section 4, "Additional Tricks"), which this form does not hold: at the start of every block
 *   of 128 columns they are rebuilt as w + s R_bb^-1 from the block's accumulators s and the inverse of the block's own
 *   128 x 128 diagonal block of R (the corrections of the waiting columns satisfy delta R_bb = s), and inside the
 *   block Alg. 1 runs on that inverse, which is the diagonal block of U.  For these group sizes the workspace also
 *   holds a copy of R with every column block scaled by that inverse (n x n floats; gptq_quantize_layer_workspace_bytes
 *   counts it whenever `group` is 32, 64 or 128).
 *   W is read in its own type at every block (it is not copied); the workspace
 *   (gptq_quantize_layer_workspace_bytes) holds the float32 accumulators instead.  All other arguments, outputs
 *   (codes, scales, zeros, Wq, half_E2_rows) and error behaviour as for gptq_quantize_layer.
 */
GPTQ_API size_t gptq_damp_cholesky_workspace_bytes(int64_t n);
GPTQ_API int gptq_damp_cholesky(float* H_R, int64_t ld, int64_t n, float percdamp,
                       void* ws, size_t ws_bytes, int* info_dev, void* stream);
GPTQ_API int gptq_quantize_layer_from_factor_supports(int64_t group);
GPTQ_API int gptq_quantize_layer_from_factor(const void* W, int wdtype, int64_t ldw, int64_t r, int64_t n,
                                    const float* R, int64_t ldr,
                                    int bits, int grid, int block, int64_t group,
                                    uint8_t* codes, int64_t ldc, float* scales, int32_t* zeros,
                                    float* Wq, int64_t ldq, double* half_E2_rows,
                                    void* ws, size_t ws_bytes, void* stream);

/*
 * The lazy batch update on its own (Alg. 1, last statement of the outer loop; Section 3, Step 2):
 *   W[r x ncols] -= E[r x k] * U[k x ncols]
 * with E the scaled errors of k already quantized columns and U the rows of the factor that belong to them,
 * restricted to the ncols columns still to be quantized -- the product gptq_quantize_layer issues after every
 * block (k = 128, the rest of the current 1024-column outer block) and after every outer block (k = 1024, all
 * later columns).  float32 on the matrix cores, float32 accumulation.  All three matrices row-major, 16-byte
 * aligned, leading dimensions multiples of 4 elements (ldw >= ncols, lde >= k, ldu >= ncols).  Any size is taken;
 * r % 256 == 0, ncols % 128 == 0 and k % 64 == 0 run on the large-tile kernel.  A zero size is a no-op.
 */
GPTQ_API int gptq_trailing_update(float* W, int64_t ldw, const float* E, int64_t lde, const float* U, int64_t ldu,
                         int64_t r, int64_t ncols, int64_t k, void* stream);

/*
 * The two deferred rank-1024 updates through split float32 products on the bf16 matrix cores -- the form
 * gptq_damp_cholesky* and gptq_quantize_layer* use for their large updates (Section 3, Steps 2 and 3; Alg. 1, last
 * statement of the outer loop).  Every float32 operand element is the exact sum of three bfloat16 pieces
 * (8 + 8 + 8 significant bits); of the nine piece products of a * b the six with i + j <= 4 are accumulated in
 * float32, smallest first; the three left out are below 2^-23 |a b|, the size of a float32 rounding.
 *
 * gptq_trailing_update_split:   W[r x ncols] -= E[r x k] * U[k x ncols]       (arguments as gptq_trailing_update)
 * gptq_symmetric_update_split:  H[n x n] -= P[n x k] * P^T on the 256 x 256 tiles that touch the upper triangle
 *                               (diagonal tiles whole; tiles below the diagonal are not written)
 *   k must be 1024 and r, ncols, n multiples of 256 (else GPTQ_ERR_UNSUPPORTED, nothing enqueued); all matrices
 *   row-major float32, 16-byte aligned, leading dimensions multiples of 4 elements.  ws: device workspace of at
 *   least *_workspace_bytes, 256-byte aligned, holds the split operands; its contents need not be initialised.
 *   Operand elements must be finite and below 2^127 in magnitude.
 */
/*
 * Which launches take the split products is decided per launch from its count of 256 x 256 tiles: at least 144.
 * gptq_set_split_min_tiles(t) with t > 0 replaces that minimum for every later call of the process (t <= 0 restores
 * it) and returns the previous setting: a tuning and test knob -- the results of a call depend on it only through
 * rounding.  Not meant to be changed while another thread is inside a library call.
 */
GPTQ_API int gptq_set_split_min_tiles(int tiles);
GPTQ_API size_t gptq_trailing_update_split_workspace_bytes(int64_t r, int64_t ncols);
GPTQ_API int gptq_trailing_update_split(float* W, int64_t ldw, const float* E, int64_t lde, const float* U, int64_t ldu,
                               int64_t r, int64_t ncols, int64_t k, void* ws, size_t ws_bytes, void* stream);
GPTQ_API size_t gptq_symmetric_update_split_workspace_bytes(int64_t n);
GPTQ_API int gptq_symmetric_update_split(float* H, int64_t ldh, const float* P, int64_t ldp, int64_t n, int64_t k,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Step 4 -- bit packing (the paper stores 3-bit weights densely, Section 4 "Practical Speedups",
 * but prints no layout; this one is ours).
 *
 *   Per row, code k occupies bits [k*bits, (k+1)*bits) of a little-endian bit stream stored as
 *   consecutive uint32 words; a code may straddle two words; the row is padded with zero bits to
 *   a whole word: words_per_row = ceil(n * bits / 32).
 *   codes [r x n] uint8 (ldc >= n), every code < 2^bits (higher bits are masked off);
 *   out   [r x ld_out] uint32, ld_out >= words_per_row.  bits in {2, 3, 4}.
 */
GPTQ_API int gptq_pack(const uint8_t* codes, int64_t ldc, int64_t r, int64_t n, int bits,
              uint32_t* out, int64_t ld_out, void* stream);
/* Inverse of gptq_pack. */
GPTQ_API int gptq_unpack(const uint32_t* words, int64_t ld_words, int64_t r, int64_t n, int bits,
                uint8_t* codes, int64_t ldc, void* stream);

/*
 * Consumers of the packed format (Section 4, "Practical Speedups"; appendix on the benchmarking setup).
 *
 *   words    [r x ld_words] uint32, the layout gptq_pack writes; scales [r x G] float32 and zeros [r x G] int32
 *            as gptq_quantize_layer writes them (G = 1 for group == 0, else n / group; n % group == 0).
 *            A weight is scale * (code - zero) with the grid of its row, or of its row's group k / group.
 *            A ternary layer is bits = 2 with zero = 1.
 *
 * gptq_dequantize_packed: the whole matrix, decompressed ahead of a large-batch product.
 *   out      [r x n] float16 or float32 (odtype = GPTQ_F16 / GPTQ_F32), ldo >= n.  The float32 product
 *            scale * (code - zero), for float16 rounded once more to nearest even.
 *
 * gptq_matvec_packed: y = Q x for one vector (batch-1 generation): weights are dequantized as they are read, the
 *   vector is not quantized.
 *   x        [n] float16 or float32 (xdtype); y [r] float32, overwritten.  Sums are accumulated in float32.
 *            group must be 0, 8, 16 or a multiple of 32.  n == 0 gives y = 0; r == 0 is a no-op.
 */
GPTQ_API int gptq_dequantize_packed(const uint32_t* words, int64_t ld_words, int64_t r, int64_t n, int bits,
                           const float* scales, const int32_t* zeros, int64_t group,
                           void* out, int odtype, int64_t ldo, void* stream);
GPTQ_API int gptq_matvec_packed(const uint32_t* words, int64_t ld_words, int64_t r, int64_t n, int bits,
                       const float* scales, const int32_t* zeros, int64_t group,
                       const void* x, int xdtype, float* y, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GPTQ_MI355_H */
