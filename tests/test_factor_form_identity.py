"""The identity the inverse-free entry points rest on, checked on the CPU against the oracle's Alg. 1.

With H + lambda I = R R^T (R upper triangular) the objective of a row is |delta R|^2, delta = w' - w.  Once columns
< j are fixed at their grid values q, the minimiser over the remaining columns makes (delta R)_k = 0 for k >= j, so
the weight Alg. 1 holds at column j when it quantizes it is

    w_j + (sum_{i<j} d_i R_ij) / R_jj,      d_i = w_i - q_i   (original weight minus final grid value),

and Alg. 1's scaled error is e_j = (that weight - q_j) * R_jj, because U = R^-1 has U_jj = 1 / R_jj
(Section 3, Step 3: the rows of Cholesky(H^-1)^T are the scaled rows of the successive inverses; Eq. 2 and Eq. 3).
A column k > j that is still waiting holds w_k + delta_k with the deltas of columns j .. k solved forward from the
same conditions, delta_k = (S_k - sum_{j<=i<k} delta_i R_ik) / R_kk with S_k = sum_{i<j} d_i R_ik: this is what a
group grid taken "from the current weights" at column j sees (groups inside a block).
The float64 emulation below follows that recurrence with lazy blocks and must give the oracle's codes, grids
and errors.  A second emulation follows the arrangement the GPU kernels use for groups inside a block (the whole
block's weights rebuilt at once through the inverse of the block's diagonal part of R) to the same bar."""
import numpy as np
import pytest

from oracle import gptq_oracle as O


def factor_form_quantize(W, R, bits, grid="minmax", block=128, group=0):
    W = np.asarray(W, dtype=np.float64)
    r, n = W.shape
    S = np.zeros((r, n))                                     # S[:, k] = sum over quantized i of d_i R_ik
    diag = np.diag(R)
    maxq = O.grid_maxq(bits, grid)
    codes = np.zeros((r, n), dtype=np.int64)
    ng = n // group if group else 1
    scales, zeros = np.zeros((r, ng)), np.zeros((r, ng), dtype=np.int64)
    E = np.zeros((r, n))
    if not group:
        scale, zero = O.grid_params(W, bits, grid)
        scales[:, 0], zeros[:, 0] = scale, zero
    for i in range(0, n, block):
        iend = min(i + block, n)
        D = np.zeros((r, iend - i))
        for j in range(i, iend):
            if group and j % group == 0:
                delta = np.zeros((r, group))                 # continuous compensation of the group's waiting columns
                for k in range(group):
                    delta[:, k] = (S[:, j + k] - delta[:, :k] @ R[j:j + k, j + k]) / diag[j + k]
                scale, zero = O.grid_params(W[:, j:j + group] + delta, bits, grid)
                scales[:, j // group], zeros[:, j // group] = scale, zero
            w_now = W[:, j] + S[:, j] / diag[j]
            codes[:, j] = O.quant_codes(w_now, scale, zero, maxq)
            q = O.dequant(codes[:, j], scale, zero)
            D[:, j - i] = W[:, j] - q
            E[:, j] = (w_now - q) * diag[j]
            S[:, j + 1:iend] += np.outer(D[:, j - i], R[j, j + 1:iend])
        S[:, iend:] += D @ R[i:iend, iend:]
    return dict(codes=codes, scale=scales, zero=zeros, E=E)


@pytest.mark.parametrize("bits,grid,group,n", [(3, "minmax", 0, 200), (4, "minmax", 32, 256), (2, "minmax", 128, 384),
                                               (2, "ternary", 128, 256), (3, "minmax", 8, 136)])
def test_factor_form_equals_algorithm_1(bits, grid, group, n):
    rng = np.random.default_rng(n + bits)
    X = rng.normal(size=(n, 6 * n)) * np.exp(0.5 * rng.normal(size=(n, 1))) + 0.4 * rng.normal(size=(1, 6 * n))
    W = (rng.normal(size=(40, n)) * 0.02).astype(np.float16).astype(np.float64)
    Hd = O.damp(O.hessian(X))
    U = O.hinv_cholesky_upper(Hd)
    R = np.linalg.cholesky(Hd[::-1, ::-1])[::-1, ::-1]       # Hd = R R^T, R upper
    assert np.allclose(R @ R.T, Hd) and np.allclose(np.tril(R, -1), 0)
    assert np.allclose(U @ R, np.eye(n), atol=1e-9)          # U = R^-1
    want = O.gptq_quantize(W, U, bits, grid, 128, group)
    got = factor_form_quantize(W, R, bits, grid, 128, group)
    assert np.array_equal(got["codes"], want["codes"])
    assert np.array_equal(got["zero"], want["zero"]) and np.allclose(got["scale"], want["scale"], rtol=1e-12)
    assert np.allclose(got["E"], want["E"], rtol=1e-6, atol=1e-9 * np.abs(want["E"]).max())


def block_form_quantize(W, R, bits, grid, group, block=128):
    """The arrangement quant_block_hybrid_kernel uses for groups inside a block: at a block start the working weights
    are w + s R_bb^-1 (the conditions (delta R)_k = 0 over the whole block), the block is then walked as Alg. 1 walks
    it, on U's diagonal block R_bb^-1, and hands d = w - q to the accumulators of the later columns."""
    W = np.asarray(W, dtype=np.float64)
    r, n = W.shape
    S = np.zeros((r, n))
    maxq = O.grid_maxq(bits, grid)
    codes = np.zeros((r, n), dtype=np.int64)
    ng = n // group
    scales, zeros = np.zeros((r, ng)), np.zeros((r, ng), dtype=np.int64)
    E = np.zeros((r, n))
    for i in range(0, n, block):
        iend = min(i + block, n)
        Ub = np.linalg.inv(R[i:iend, i:iend])
        Wb = W[:, i:iend] + S[:, i:iend] @ Ub                # the block's weights as they stand now
        D = np.zeros((r, iend - i))
        for j in range(i, iend):
            c = j - i
            if j % group == 0:
                scale, zero = O.grid_params(Wb[:, c:c + group], bits, grid)
                scales[:, j // group], zeros[:, j // group] = scale, zero
            codes[:, j] = O.quant_codes(Wb[:, c], scale, zero, maxq)
            q = O.dequant(codes[:, j], scale, zero)
            E[:, j] = (Wb[:, c] - q) / Ub[c, c]
            Wb[:, c + 1:] -= np.outer(E[:, j], Ub[c, c + 1:])
            D[:, c] = W[:, j] - q
        S[:, iend:] += D @ R[i:iend, iend:]
    return dict(codes=codes, scale=scales, zero=zeros, E=E)


@pytest.mark.parametrize("bits,grid,group,n", [(4, "minmax", 32, 416), (2, "minmax", 128, 384), (2, "ternary", 64, 320)])
def test_block_form_with_group_grids_equals_algorithm_1(bits, grid, group, n):
    rng = np.random.default_rng(7 * n + bits)
    X = rng.normal(size=(n, 6 * n)) * np.exp(0.5 * rng.normal(size=(n, 1))) + 0.4 * rng.normal(size=(1, 6 * n))
    W = (rng.normal(size=(24, n)) * 0.02).astype(np.float16).astype(np.float64)
    Hd = O.damp(O.hessian(X))
    U = O.hinv_cholesky_upper(Hd)
    R = np.linalg.cholesky(Hd[::-1, ::-1])[::-1, ::-1]
    want = O.gptq_quantize(W, U, bits, grid, 128, group)
    got = block_form_quantize(W, R, bits, grid, group)
    assert np.array_equal(got["codes"], want["codes"])
    assert np.array_equal(got["zero"], want["zero"]) and np.allclose(got["scale"], want["scale"], rtol=1e-10)
    assert np.allclose(got["E"], want["E"], rtol=1e-6, atol=1e-9 * np.abs(want["E"]).max())
