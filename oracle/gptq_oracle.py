"""Float64 CPU oracle for the GPTQ per-layer solver (Frantar et al., arXiv 2210.17323).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, step-by-step NumPy
implementation of what the GPU path must compute.  It shares no code with the HIP library and
must only be imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.

GPTQ is a heuristic (it does not reach the minimiser of the layer-wise objective, Eq. 1), so the
oracle follows the algorithm's steps in the paper's order and notation:

  hessian                      H = 2 X X^T                      (Section 2, text before Eq. 2; Alg. 1 caption)
  damp                         H + lambda I, lambda = 1% of mean(diag H)   (Section 3, Step 3)
  hinv_cholesky_upper          U = Cholesky(H^-1)^T             (Alg. 1, third statement)
  gptq_quantize                the block / column double loop   (Alg. 1)
  naive_obs_quantize           Eq. 2 update + Eq. 3 downdate per column, fixed order (Section 3, Step 1)
  rtn_quantize                 round-to-nearest on the same grid (Section 4, Baselines)
  brute_force_row_error        exhaustive minimum of Eq. 1 for one short row
  minmax_grid / ternary_grid   the quantization grids           (Section 4, Setup; "Extreme Quantization")
  pack_codes / unpack_codes    dense b-bit stream               (layout is this build's; the paper gives none)

Arithmetic is float64 throughout, including the one place where floating point decides an integer:
the grid parameters (scale, zero point) and the rounding w -> code.  `decision_dtype=np.float32`
evaluates just that decision (the grid parameters and w/scale) in float32 instead, the precision in
which a float32 implementation takes it; everything else stays float64.  Tests compare the GPU path
with both variants.

Pins (tests/test_oracle_*.py): diagonal H reduces to RTN exactly; the blocked Cholesky form equals
the naive Eq. 2 + Eq. 3 procedure; codes lie on the grid; brute force on <= 6 columns is never
worse; block-size / row-subset / H-scaling invariance; W0 - Q = E U and the closed-form layer
error; U^T U (H + lambda I) = I, literal route == reverse-order route, corner property, Eq. 3 row
identity; Hessian exact on small integers; packing against hand-computed words.
`ternary_grid` is *parity unpinned by the paper* (the paper only names the levels -1, 0, +1; the
choice of the scale s = max|w| is this build's reading).
"""
from __future__ import annotations

import itertools

import numpy as np


# --------------------------------------------------------------------------------------------
# Hessian, damping, Cholesky of the inverse
# --------------------------------------------------------------------------------------------

def hessian(X) -> np.ndarray:
    """H = 2 X X^T for X of shape (d_col, tokens).  Section 2: the Hessian of the per-row
    quadratic objective; Alg. 1 caption."""
    X = np.asarray(X, dtype=np.float64)
    return 2.0 * (X @ X.T)


def damping_lambda(H, percdamp: float = 0.01) -> float:
    """lambda = percdamp * mean(diag H): "1% of the average diagonal value" (Section 3, Step 3)."""
    return float(percdamp) * float(np.mean(np.diag(np.asarray(H, dtype=np.float64))))


def damp(H, percdamp: float = 0.01) -> np.ndarray:
    """H + lambda I (Alg. 1 caption)."""
    Hd = np.array(H, dtype=np.float64, copy=True)
    Hd[np.diag_indices_from(Hd)] += damping_lambda(H, percdamp)
    return Hd


def hinv_cholesky_upper(Hd) -> np.ndarray:
    """U = Cholesky(Hd^-1)^T: invert, take the lower Cholesky factor L of the inverse, transpose.
    U is upper triangular with Hd^-1 = U^T U (Alg. 1, third statement)."""
    Hinv = np.linalg.inv(np.asarray(Hd, dtype=np.float64))
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv).T.copy()


def hinv_cholesky_upper_reverse(Hd) -> np.ndarray:
    """The same U by a different route (used as a cross-check): factor Hd = R R^T with R upper
    triangular -- a Cholesky factorisation taken in reversed index order -- then U = R^-1, because
    Hd^-1 = R^-T R^-1 and the Cholesky factor with positive diagonal is unique."""
    Hd = np.asarray(Hd, dtype=np.float64)
    Lrev = np.linalg.cholesky(Hd[::-1, ::-1])
    R = Lrev[::-1, ::-1]
    n = Hd.shape[0]
    import scipy.linalg
    return scipy.linalg.solve_triangular(R, np.eye(n), lower=False)


# --------------------------------------------------------------------------------------------
# Grids
# --------------------------------------------------------------------------------------------

def minmax_grid(w, bits: int, decision_dtype=np.float64, with_real_zero: bool = False):
    """Uniform asymmetric min-max grid for each row of w (Section 4, Setup).

    The range is widened to contain 0 so that an integer zero point in [0, maxq] exists:
      lo = min(min w, 0), hi = max(max w, 0), scale = (hi - lo)/maxq, zero = rint(-lo/scale),
    and an all-zero row gets scale 1, zero 0.  Returns (scale[rows] decision_dtype, zero[rows] int64), and with
    with_real_zero also the value -lo/scale before it is rounded (for reporting how close to a tie it was).
    """
    w = np.asarray(w).astype(decision_dtype)
    maxq = decision_dtype(2 ** bits - 1)
    lo = np.minimum(w.min(axis=1), decision_dtype(0))
    hi = np.maximum(w.max(axis=1), decision_dtype(0))
    dead = hi == lo
    scale = (hi - lo) / maxq
    scale[dead] = decision_dtype(1)
    real_zero = -lo / scale
    zero = np.rint(real_zero)
    zero[dead] = 0
    if with_real_zero:
        return scale.astype(decision_dtype), zero.astype(np.int64), np.asarray(real_zero, dtype=np.float64)
    return scale.astype(decision_dtype), zero.astype(np.int64)


def ternary_grid(w, decision_dtype=np.float64):
    """Levels {-s, 0, +s} with s = max|w| per row (s = 1 for an all-zero row), stored as codes
    {0, 1, 2} with zero point 1 ("Extreme Quantization" names the levels; the scale is our reading)."""
    w = np.asarray(w).astype(decision_dtype)
    s = np.abs(w).max(axis=1)
    s[s == 0] = decision_dtype(1)
    return s.astype(decision_dtype), np.ones(w.shape[0], dtype=np.int64)


def grid_params(w, bits: int, grid: str, decision_dtype=np.float64):
    if grid == "minmax":
        return minmax_grid(w, bits, decision_dtype)
    if grid == "ternary":
        return ternary_grid(w, decision_dtype)
    raise ValueError(grid)


def grid_maxq(bits: int, grid: str) -> int:
    return 2 if grid == "ternary" else 2 ** bits - 1


def quant_codes(w, scale, zero, maxq: int, decision_dtype=np.float64) -> np.ndarray:
    """quant(w): index of the nearest grid value, code = clamp(rint(w/scale) + zero, 0, maxq),
    ties to even (Section 2: quant rounds to the nearest value on the grid)."""
    x = np.asarray(w).astype(decision_dtype) / np.asarray(scale, dtype=decision_dtype)
    return np.clip(np.rint(x).astype(np.int64) + zero, 0, maxq)


def dequant(codes, scale, zero) -> np.ndarray:
    """Grid value of a code: scale * (code - zero), in float64."""
    return np.asarray(scale, dtype=np.float64) * (np.asarray(codes, dtype=np.float64) - zero)


# --------------------------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------------------------

def gptq_quantize(W, U, bits: int, grid: str = "minmax", block: int = 128, group: int = 0,
                  decision_dtype=np.float64, teacher_codes=None, teacher_levels=None):
    """Algorithm 1: quantize W (d_row x d_col) given U = Cholesky(H^-1)^T and block size B.

    group == 0: one grid per row, fixed from the original weights before the process starts
    (Section 2: the grid is fixed beforehand).  group == g > 0: a new grid for columns
    [j, j+g) whenever j is a multiple of g, found from the *current* (already updated) weights
    (Section 4, "175 Billion Parameter Models": group parameters use the most current weights).
    Because updates to columns beyond the current block are deferred, "current" is only well
    defined when no group straddles a block end: B must be a multiple of g or g a multiple of B.

    teacher_codes (optional, d_row x d_col): "teacher forcing" for comparing two arithmetics without the
    avalanche that follows a single differing rounding decision.  The code this function would choose
    for each column is still computed from the current weights and returned as `codes`, but the
    algorithm then continues with the teacher's code (Q, E and all updates use it), so every decision
    is taken on the teacher's history.  In grouped mode the grids are still computed here.
    teacher_levels gives the teacher's decisions as grid levels (code - zero point) instead: the forced
    code is level + this function's own zero point, so the forced grid VALUE is the teacher's even where
    the two zero points differ by a tie of rint(-lo/scale).

    Returns a dict with codes (int64), scale (rows x groups, decision_dtype), zero (int64),
    Q (float64 dequantised weights), E (d_row x d_col, every column's scaled error),
    W_final (the working copy after all updates), frac (the pre-rounding values w/scale) and zero_real
    (rows x groups, the pre-rounding zero points -lo/scale of the min-max grid).
    U may be float32 (it is widened to float64 block row by block row).
    """
    Wk = np.array(W, dtype=np.float64, copy=True)
    U = np.asarray(U)
    r, n = Wk.shape
    if group and n % group:
        raise ValueError("d_col must be a multiple of the group size")
    if group and block % group and group % block:
        # a group that straddles a block end would take its grid from columns that the lazy
        # trailing update has not reached yet, i.e. not from the current weights
        raise ValueError("group boundaries must align with block boundaries")
    maxq = grid_maxq(bits, grid)
    ngroups = n // group if group else 1
    scales = np.zeros((r, ngroups), dtype=decision_dtype)
    zeros = np.zeros((r, ngroups), dtype=np.int64)
    Q = np.zeros((r, n))
    codes = np.zeros((r, n), dtype=np.int64)
    E_all = np.zeros((r, n))
    zero_real = np.full((r, ngroups), np.nan)        # -lo/scale before rounding (min-max grid; reporting only)
    if not group:
        scale, zero = grid_params(Wk, bits, grid, decision_dtype)
        scales[:, 0], zeros[:, 0] = scale, zero
        if grid == "minmax":
            zero_real[:, 0] = minmax_grid(Wk, bits, decision_dtype, with_real_zero=True)[2]
    frac = np.zeros((r, n), dtype=decision_dtype)
    for i in range(0, n, block):
        iend = min(i + block, n)
        E = np.zeros((r, iend - i))
        Ub = np.asarray(U[i:iend], dtype=np.float64)        # rows i..iend-1 of U, exact widening
        for j in range(i, iend):
            if group and j % group == 0:
                scale, zero = grid_params(Wk[:, j:j + group], bits, grid, decision_dtype)
                scales[:, j // group], zeros[:, j // group] = scale, zero
                if grid == "minmax":
                    zero_real[:, j // group] = minmax_grid(Wk[:, j:j + group], bits, decision_dtype, with_real_zero=True)[2]
            codes[:, j] = quant_codes(Wk[:, j], scale, zero, maxq, decision_dtype)
            frac[:, j] = Wk[:, j].astype(decision_dtype) / scale
            if teacher_levels is not None:
                used = np.asarray(teacher_levels)[:, j].astype(np.int64) + zero
            elif teacher_codes is not None:
                used = np.asarray(teacher_codes)[:, j].astype(np.int64)
            else:
                used = codes[:, j]
            Q[:, j] = dequant(used, scale, zero)
            E[:, j - i] = (Wk[:, j] - Q[:, j]) / Ub[j - i, j]
            Wk[:, j:iend] -= np.outer(E[:, j - i], Ub[j - i, j:iend])
        Wk[:, iend:] -= E @ Ub[:, iend:]
        E_all[:, i:iend] = E
    return dict(codes=codes, scale=scales, zero=zeros, Q=Q, E=E_all, W_final=Wk, frac=frac, zero_real=zero_real)


def naive_obs_quantize(W, Hd, bits: int, grid: str = "minmax", group: int = 0, decision_dtype=np.float64):
    """Fixed-order OBQ without Cholesky and without blocks (Section 3, Step 1): for each column q in
    natural order, quantize it, apply Eq. 2's update with column q of the explicit inverse Hessian of
    the remaining set F, then remove q from the inverse by the Gaussian-elimination step of Eq. 3."""
    Wk = np.array(W, dtype=np.float64, copy=True)
    r, n = Wk.shape
    maxq = grid_maxq(bits, grid)
    ngroups = n // group if group else 1
    scales = np.zeros((r, ngroups), dtype=decision_dtype)
    zeros = np.zeros((r, ngroups), dtype=np.int64)
    Q = np.zeros((r, n))
    codes = np.zeros((r, n), dtype=np.int64)
    if not group:
        scale, zero = grid_params(Wk, bits, grid, decision_dtype)
        scales[:, 0], zeros[:, 0] = scale, zero
    Hinv = np.linalg.inv(np.asarray(Hd, dtype=np.float64))      # inverse Hessian of F = {q, ..., n-1}
    for q in range(n):
        if group and q % group == 0:
            scale, zero = grid_params(Wk[:, q:q + group], bits, grid, decision_dtype)
            scales[:, q // group], zeros[:, q // group] = scale, zero
        codes[:, q] = quant_codes(Wk[:, q], scale, zero, maxq, decision_dtype)
        Q[:, q] = dequant(codes[:, q], scale, zero)
        # Eq. 2: delta_F = -(w_q - quant(w_q)) / [Hinv]_qq * Hinv[:, q]; position 0 of Hinv is q
        delta = -np.outer((Wk[:, q] - Q[:, q]) / Hinv[0, 0], Hinv[:, 0])
        Wk[:, q:] += delta
        # Eq. 3: eliminate q, then drop its row and column
        Hinv = (Hinv - np.outer(Hinv[:, 0], Hinv[0, :]) / Hinv[0, 0])[1:, 1:]
    return dict(codes=codes, scale=scales, zero=zeros, Q=Q)


def rtn_quantize(W, bits: int, grid: str = "minmax", group: int = 0, decision_dtype=np.float64):
    """Round every weight to the nearest value of the same grid (Section 4, Baselines)."""
    W = np.asarray(W, dtype=np.float64)
    r, n = W.shape
    g = group if group else n
    maxq = grid_maxq(bits, grid)
    codes = np.zeros((r, n), dtype=np.int64)
    Q = np.zeros((r, n))
    scales = np.zeros((r, n // g), dtype=decision_dtype)
    zeros = np.zeros((r, n // g), dtype=np.int64)
    for k in range(n // g):
        sl = slice(k * g, (k + 1) * g)
        scale, zero = grid_params(W[:, sl], bits, grid, decision_dtype)
        scales[:, k], zeros[:, k] = scale, zero
        codes[:, sl] = quant_codes(W[:, sl], scale[:, None], zero[:, None], maxq, decision_dtype)
        Q[:, sl] = dequant(codes[:, sl], scale[:, None], zero[:, None])
    return dict(codes=codes, scale=scales, zero=zeros, Q=Q)


# --------------------------------------------------------------------------------------------
# Errors
# --------------------------------------------------------------------------------------------

def layer_error_X(W, Q, X) -> float:
    """||W X - Q X||_F^2, the objective of Eq. 1."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(Q, dtype=np.float64)
    return float(np.sum((D @ np.asarray(X, dtype=np.float64)) ** 2))


def layer_error_H(W, Q, H) -> float:
    """The same objective through the Hessian: (1/2) tr(D H D^T) with H = 2 X X^T, D = W - Q."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(Q, dtype=np.float64)
    return 0.5 * float(np.sum((D @ np.asarray(H, dtype=np.float64)) * D))


def row_errors_H(W, Q, H) -> np.ndarray:
    D = np.asarray(W, dtype=np.float64) - np.asarray(Q, dtype=np.float64)
    return 0.5 * np.sum((D @ np.asarray(H, dtype=np.float64)) * D, axis=1)


def brute_force_row_error(w, H, scale, zero, maxq: int) -> float:
    """min over all (maxq+1)^n grid points q of (1/2)(w-q)^T H (w-q) for one short row."""
    w = np.asarray(w, dtype=np.float64)
    H = np.asarray(H, dtype=np.float64)
    levels = float(scale) * (np.arange(maxq + 1, dtype=np.float64) - float(zero))
    best = np.inf
    for combo in itertools.product(levels, repeat=w.shape[0]):
        d = w - np.array(combo)
        best = min(best, 0.5 * float(d @ H @ d))
    return best


# --------------------------------------------------------------------------------------------
# Packing and storage cost
# --------------------------------------------------------------------------------------------

def packed_words_per_row(n: int, bits: int) -> int:
    return (n * bits + 31) // 32


def pack_codes(codes, bits: int) -> np.ndarray:
    """Row-wise dense bit stream: code k of a row occupies bits [k*b, (k+1)*b) of the row's
    little-endian stream of uint32 words (a code may straddle two words); rows are padded with
    zero bits to a whole word."""
    codes = np.asarray(codes)
    r, n = codes.shape
    if codes.size and (codes.min() < 0 or codes.max() >= (1 << bits)):
        raise ValueError("code out of range")
    nwords = packed_words_per_row(n, bits)
    # bit t of code k goes to stream position k*bits + t
    bitplane = ((codes.astype(np.uint8)[:, :, None] >> np.arange(bits, dtype=np.uint8)) & 1).reshape(r, n * bits)
    stream = np.zeros((r, nwords * 32), dtype=np.uint8)
    stream[:, :n * bits] = bitplane
    by = np.packbits(stream, axis=1, bitorder="little")           # byte i holds stream bits 8i..8i+7
    return np.ascontiguousarray(by).view("<u4").astype(np.uint32).reshape(r, nwords)


def unpack_codes(words, n: int, bits: int) -> np.ndarray:
    """Inverse of pack_codes."""
    words = np.ascontiguousarray(np.asarray(words, dtype="<u4"))
    r = words.shape[0]
    stream = np.unpackbits(words.view(np.uint8).reshape(r, -1), axis=1, bitorder="little")[:, :n * bits]
    weights = (1 << np.arange(bits)).astype(np.int64)
    return (stream.reshape(r, n, bits).astype(np.int64) * weights).sum(axis=2)


def dequantize_packed(words, n: int, bits: int, scale, zero, group: int = 0) -> np.ndarray:
    """The weight matrix a packed layer stands for: entry (i, k) is scale * (code - zero) with the
    scale and zero point of row i (group == 0) or of row i's group k // group (Section 4, "Practical
    Speedups": weights are dequantized when they are needed).  float64."""
    codes = unpack_codes(words, n, bits)
    scale = np.asarray(scale, dtype=np.float64)
    zero = np.asarray(zero, dtype=np.float64)
    if group:
        scale = np.repeat(scale, group, axis=1)[:, :n]
        zero = np.repeat(zero, group, axis=1)[:, :n]
    return scale * (codes - zero)


def matvec_packed(words, n: int, bits: int, scale, zero, group: int, x) -> np.ndarray:
    """Quantized-matrix times full-precision vector (Section 4, "Practical Speedups"): y = Q x with
    Q the dequantized matrix; the vector is not quantized.  float64."""
    return dequantize_packed(words, n, bits, scale, zero, group) @ np.asarray(x, dtype=np.float64)


def bits_per_weight(bits: int, group: int, scale_bits: int = 16) -> float:
    """Average storage per weight for a grouped grid holding one scale of scale_bits and one
    bits-wide integer zero point per group ("Extreme Quantization": FP16 scale and 2-bit zero
    point per group of 128 is about 2.2 bits)."""
    return bits + (scale_bits + bits) / group
