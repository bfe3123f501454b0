"""Pins for the CPU oracle: each test checks the oracle against something other than itself --
closed forms, special cases that reduce to a textbook routine, identities the paper states,
brute force on tiny inputs, and the storage figures the paper prints.  CPU only."""
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import gptq_oracle as O
from workloads import configs


def _small_layer(r=24, n=40, m=160, seed_shift=0, kind="lognormal"):
    base = configs.config2()[0] if kind == "lognormal" else configs.config3()[1]
    lay = configs.scaled_twin(base, n, r=r, m=m)
    lay = type(lay)(**{**lay.__dict__, "tensor_id": lay.tensor_id + seed_shift,
                       "x": type(lay.x)(**{**lay.x.__dict__, "tensor_id": lay.x.tensor_id + seed_shift})})
    W = lay.weights().double().numpy()
    X = lay.x.tile().double().numpy()
    return W, X


def _solve(W, X, **kw):
    H = O.hessian(X)
    Hd = O.damp(H)
    U = O.hinv_cholesky_upper(Hd)
    return H, Hd, U, O.gptq_quantize(W, U, **kw)


# ------------------------------------------------------------------ Hessian

def test_hessian_exact_on_small_integers():
    rng = np.random.default_rng(0)
    X = rng.integers(-7, 8, size=(9, 33))
    want = np.zeros((9, 9), dtype=np.int64)
    for a in range(9):
        for b in range(9):
            want[a, b] = 2 * sum(int(X[a, t]) * int(X[b, t]) for t in range(33))
    H = O.hessian(X)
    assert (H == want).all()
    assert (H == H.T).all()
    assert np.linalg.eigvalsh(H).min() > -1e-9


def test_hessian_is_hessian_of_the_objective():
    # second derivative of f(w) = ||w X - w0 X||^2 along random directions is d^T H d
    W, X = _small_layer(1, 12, 50)
    H = O.hessian(X)
    rng = np.random.default_rng(1)
    w0 = W[0]
    f = lambda w: float(np.sum(((w - w0) @ X) ** 2))
    for _ in range(3):
        d = rng.standard_normal(12)
        second = f(w0 + d) - 2 * f(w0) + f(w0 - d)       # exact for a quadratic
        assert np.isclose(second, d @ H @ d, rtol=1e-10)


def test_damping_is_one_percent_of_mean_diagonal():
    H = np.diag([1.0, 2.0, 3.0, 6.0])
    Hd = O.damp(H, 0.01)
    assert np.allclose(np.diag(Hd) - np.diag(H), 0.03)
    assert np.allclose(Hd - np.diag(np.diag(Hd)), 0)


# ------------------------------------------------------------------ U = Cholesky(H^-1)^T

def test_U_defining_identity_and_routes():
    _, X = _small_layer(1, 48, 200)
    Hd = O.damp(O.hessian(X))
    U = O.hinv_cholesky_upper(Hd)
    assert np.allclose(np.tril(U, -1), 0) and (np.diag(U) > 0).all()
    assert np.allclose(U.T @ U @ Hd, np.eye(48), atol=1e-9)
    U2 = O.hinv_cholesky_upper_reverse(Hd)
    assert np.allclose(U, U2, rtol=1e-9, atol=1e-14)
    # closed form for the last pivot and the corner property
    assert np.isclose(U[-1, -1], Hd[-1, -1] ** -0.5)
    for k in (1, 17, 40):
        assert np.allclose(U[k:, k:], O.hinv_cholesky_upper(Hd[k:, k:]), rtol=1e-9, atol=1e-14)


def test_U_diagonal_hessian():
    h = np.array([4.0, 0.25, 9.0, 1.0])
    U = O.hinv_cholesky_upper(np.diag(h))
    assert np.allclose(U, np.diag(h ** -0.5))


def test_U_rows_are_scaled_rows_of_the_downdated_inverse():
    # Section 3, Step 3: row q of Hinv_{F_q} from the diagonal on, divided by sqrt of its diagonal
    # entry, is row q of U; Hinv_{F_q} obtained by q elimination steps of Eq. 3.
    _, X = _small_layer(1, 10, 64)
    Hd = O.damp(O.hessian(X))
    U = O.hinv_cholesky_upper(Hd)
    Hinv = np.linalg.inv(Hd)
    for q in range(10):
        assert np.allclose(Hinv, np.linalg.inv(Hd[q:, q:]), rtol=1e-8)      # Eq. 3 really is the inverse of H_F
        assert np.allclose(U[q, q:], Hinv[0, :] / np.sqrt(Hinv[0, 0]), rtol=1e-9)
        Hinv = (Hinv - np.outer(Hinv[:, 0], Hinv[0, :]) / Hinv[0, 0])[1:, 1:]


# ------------------------------------------------------------------ grids

def test_minmax_grid_closed_form():
    w = np.array([[-1.0, 0.5, 2.0], [0.25, 0.5, 1.0], [-3.0, -2.0, -1.0], [0.0, 0.0, 0.0]])
    scale, zero = O.minmax_grid(w, 2)
    assert np.allclose(scale, [1.0, 1.0 / 3.0, 1.0, 1.0])
    assert list(zero) == [1, 0, 3, 0]
    codes = O.quant_codes(w, scale[:, None], zero[:, None], 3)
    assert codes.tolist() == [[0, 1, 3], [1, 2, 3], [0, 1, 2], [0, 0, 0]]   # 0.5/1 -> rint(0.5) = 0, + zero 1
    q = O.dequant(codes, scale[:, None], zero[:, None])
    assert np.allclose(q[0], [-1.0, 0.0, 2.0])
    # extreme values of every row are reproduced exactly when 0 is inside the range
    assert q[0].min() == -1.0 and q[0].max() == 2.0


def test_rounding_is_half_to_even():
    scale = np.array([1.0], dtype=np.float32)
    c = O.quant_codes(np.array([0.5, 1.5, 2.5, 3.5]), scale, np.array([0]), 15)
    assert c.tolist() == [0, 2, 2, 4]


def test_ternary_grid():
    w = np.array([[0.9, -0.2, -2.0, 1.1], [0.0, 0.0, 0.0, 0.0]])
    s, z = O.ternary_grid(w)
    assert np.allclose(s, [2.0, 1.0]) and list(z) == [1, 1]
    codes = O.quant_codes(w, s[:, None], z[:, None], 2)
    assert codes.tolist() == [[1, 1, 0, 2], [1, 1, 1, 1]]
    assert np.allclose(O.dequant(codes, s[:, None], z[:, None])[0], [0, 0, -2.0, 2.0])


# ------------------------------------------------------------------ Algorithm 1

@pytest.mark.parametrize("bits,grid,group", [(4, "minmax", 0), (3, "minmax", 0), (2, "minmax", 8), (2, "ternary", 8)])
def test_diagonal_hessian_reduces_to_rtn(bits, grid, group):
    W, _ = _small_layer(16, 32, 64)
    rng = np.random.default_rng(3)
    Hd = np.diag(rng.uniform(0.5, 4.0, size=32))
    U = O.hinv_cholesky_upper(Hd)
    got = O.gptq_quantize(W, U, bits, grid, block=8, group=group)
    want = O.rtn_quantize(W, bits, grid, group)
    assert (got["codes"] == want["codes"]).all()
    assert (got["scale"] == want["scale"]).all() and (got["zero"] == want["zero"]).all()
    assert np.array_equal(got["Q"], want["Q"])


@pytest.mark.parametrize("bits,grid,group,block", [(4, "minmax", 0, 16), (3, "minmax", 0, 128), (2, "minmax", 8, 16),
                                                   (2, "ternary", 8, 16), (3, "minmax", 20, 20), (4, "minmax", 20, 10)])
def test_blocked_cholesky_form_equals_naive_obs(bits, grid, group, block):
    W, X = _small_layer(12, 40, 200, seed_shift=bits)
    H, Hd, U, got = _solve(W, X, bits=bits, grid=grid, block=block, group=group)
    want = O.naive_obs_quantize(W, Hd, bits, grid, group)
    assert (got["codes"] == want["codes"]).all()
    assert (got["zero"] == want["zero"]).all()
    assert np.allclose(got["scale"], want["scale"], rtol=1e-6)
    assert np.allclose(got["Q"], want["Q"], rtol=1e-6, atol=1e-12)


@pytest.mark.parametrize("bits,grid,group", [(4, "minmax", 0), (3, "minmax", 0), (2, "minmax", 16), (2, "ternary", 16)])
def test_codes_on_grid_and_Q_consistent(bits, grid, group):
    W, X = _small_layer(20, 48, 256)
    _, _, _, out = _solve(W, X, bits=bits, grid=grid, block=16, group=group)
    maxq = O.grid_maxq(bits, grid)
    c = out["codes"]
    assert c.dtype == np.int64 and c.min() >= 0 and c.max() <= maxq
    g = group if group else 48
    scale = np.repeat(out["scale"].astype(np.float64), g, axis=1)
    zero = np.repeat(out["zero"], g, axis=1)
    assert np.array_equal(out["Q"], scale * (c - zero))
    assert (out["zero"] >= 0).all() and (out["zero"] <= maxq).all()
    assert c.max() == maxq and c.min() == 0          # the grid is actually used end to end


def test_brute_force_is_never_worse_and_gptq_beats_rtn():
    tot_g = tot_r = tot_b = 0.0
    for shift, n in ((0, 4), (1, 5), (2, 6)):
        W, X = _small_layer(6, n, 64, seed_shift=shift)
        H, Hd, U, out = _solve(W, X, bits=2, block=128)
        rt = O.rtn_quantize(W, 2)
        eg = O.row_errors_H(W, out["Q"], Hd)
        er = O.row_errors_H(W, rt["Q"], Hd)
        for row in range(6):
            eb = O.brute_force_row_error(W[row], Hd, out["scale"][row, 0], out["zero"][row, 0], 3)
            assert eb <= eg[row] * (1 + 1e-12) + 1e-18
            assert eb <= er[row] * (1 + 1e-12) + 1e-18
            tot_b += eb
        tot_g += eg.sum()
        tot_r += er.sum()
    assert tot_b <= tot_g < tot_r


def test_group_must_not_straddle_a_block_end():
    W, X = _small_layer(4, 40, 100)
    U = O.hinv_cholesky_upper(O.damp(O.hessian(X)))
    with pytest.raises(ValueError):
        O.gptq_quantize(W, U, 2, block=12, group=8)
    with pytest.raises(ValueError):
        O.gptq_quantize(W, U, 2, block=16, group=7)


def test_block_size_invariance():
    W, X = _small_layer(16, 64, 300)
    H = O.hessian(X)
    U = O.hinv_cholesky_upper(O.damp(H))
    ref = O.gptq_quantize(W, U, 3, block=64)
    for B in (1, 5, 32, 128):
        out = O.gptq_quantize(W, U, 3, block=B)
        assert (out["codes"] == ref["codes"]).all()
        assert np.allclose(out["E"], ref["E"], rtol=1e-8, atol=1e-12)


def test_row_subset_and_hessian_scaling_invariance():
    W, X = _small_layer(16, 48, 256)
    H = O.hessian(X)
    U = O.hinv_cholesky_upper(O.damp(H))
    full = O.gptq_quantize(W, U, 4, block=16)
    sub = O.gptq_quantize(W[3:9], U, 4, block=16)
    assert (sub["codes"] == full["codes"][3:9]).all()
    U7 = O.hinv_cholesky_upper(O.damp(7.0 * H))
    assert np.allclose(U7, U / np.sqrt(7.0), rtol=1e-10)
    sc = O.gptq_quantize(W, U7, 4, block=16)
    assert (sc["codes"] == full["codes"]).all()


def test_error_identities():
    # W0 - Q = E U  and  (1/2) tr(D Hd D^T) = (1/2) ||E||_F^2   (each step is the exact constrained
    # minimiser of the quadratic, so the per-step losses (1/2) e^2 / [Hinv_F]_qq add up)
    W, X = _small_layer(16, 48, 256, kind="relu")
    H, Hd, U, out = _solve(W, X, bits=3, block=16)
    assert np.allclose(W - out["Q"], out["E"] @ U, rtol=1e-9, atol=1e-13)
    assert np.isclose(O.layer_error_H(W, out["Q"], Hd), 0.5 * np.sum(out["E"] ** 2), rtol=1e-9)
    assert np.isclose(O.layer_error_H(W, out["Q"], H), O.layer_error_X(W, out["Q"], X), rtol=1e-9)
    # the working copy ends up equal to Q (every column is overwritten by its own update)
    assert np.allclose(out["W_final"], out["Q"], atol=1e-12)


def test_first_column_is_rtn_and_error_beats_rtn():
    W, X = _small_layer(32, 64, 512)
    H, Hd, U, out = _solve(W, X, bits=3, block=32)
    rt = O.rtn_quantize(W, 3)
    assert (out["codes"][:, 0] == rt["codes"][:, 0]).all()
    assert O.layer_error_X(W, out["Q"], X) < O.layer_error_X(W, rt["Q"], X)
    # correlated inputs (non-zero-mean, post-ReLU-like) are where error compensation pays most
    W, X = _small_layer(32, 64, 512, kind="relu")
    H, Hd, U, out = _solve(W, X, bits=3, block=32)
    assert O.layer_error_X(W, out["Q"], X) < 0.85 * O.layer_error_X(W, O.rtn_quantize(W, 3)["Q"], X)


def test_one_obs_step_is_the_constrained_minimiser():
    # Eq. 2: after fixing w_0 to its grid value, the updated remaining weights minimise the quadratic.
    W, X = _small_layer(1, 8, 64)
    H, Hd, U, _ = _solve(W, X, bits=3)
    w = W[0]
    scale, zero = O.minmax_grid(W, 3)
    q0 = O.dequant(O.quant_codes(w[0], scale[0], zero[0], 7), scale[0], zero[0])
    # minimise (1/2)(v-w)^T Hd (v-w) subject to v_0 = q0:  v_rest = w_rest - Hd_rr^-1 Hd_r0 (q0 - w_0)
    v_rest = w[1:] - np.linalg.solve(Hd[1:, 1:], Hd[1:, 0]) * (q0 - w[0])
    e = (w[0] - q0) / U[0, 0]
    assert np.allclose(w[1:] - e * U[0, 1:], v_rest, rtol=1e-9, atol=1e-14)


# ------------------------------------------------------------------ packing and storage

def test_pack_hand_computed_words():
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3]])
    # 3-bit: word0 = 1 + (2<<3) + (3<<6) + (4<<9) + (5<<12) + (6<<15) + (7<<18) + (0<<21) + (1<<24) + (2<<27)
    #               + ((3 & 0b11) << 30);  word1 = 3 >> 2 = 0
    assert O.pack_codes(codes, 3).tolist() == [[0xD11F58D1, 0x0]]
    codes[0, 10] = 7                        # 0b111: low two bits in word0 (unchanged), high bit in word1
    assert O.pack_codes(codes, 3).tolist() == [[0xD11F58D1, 0x1]]
    assert O.pack_codes(np.array([[3, 0, 1, 2] * 4 + [2]]), 2).tolist() == [[0x93939393, 0x2]]
    assert O.pack_codes(np.array([[0xF, 0x1, 0x0, 0xA, 0x5, 0x5, 0x0, 0x8]]), 4).tolist() == [[0x8055A01F]]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_round_trip(bits):
    rng = np.random.default_rng(bits)
    for n in (1, 31, 32, 33, 127, 200):
        codes = rng.integers(0, 1 << bits, size=(5, n))
        words = O.pack_codes(codes, bits)
        assert words.shape == (5, (n * bits + 31) // 32) and words.dtype == np.uint32
        assert (O.unpack_codes(words, n, bits) == codes).all()
    with pytest.raises(ValueError):
        O.pack_codes(np.array([[1 << bits]]), bits)


def test_storage_bits_match_paper_figures():
    path = os.path.join(os.path.dirname(__file__), "golden", "storage_bits.txt")
    rows = [ln.split(None, 5) for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 4
    for bits, group, what, value, tol, _cite in rows:
        total = O.bits_per_weight(int(bits), int(group))
        got = total if what == "total" else total - int(bits)
        assert abs(got - float(value)) <= float(tol), (bits, group, got)


def test_teacher_forcing_reproduces_own_decisions_and_isolates_a_flip():
    W, X = _small_layer(8, 64, 300)
    H, Hd, U, ref = _solve(W, X, bits=3, block=16)
    # forcing the oracle with its own codes changes nothing
    same = O.gptq_quantize(W, U, 3, block=16, teacher_codes=ref["codes"])
    assert (same["codes"] == ref["codes"]).all() and np.array_equal(same["Q"], ref["Q"])
    # a teacher that differs in one early code: the oracle flags exactly that column as its own different
    # choice, follows the teacher's history afterwards, and its Q equals the teacher's codes on the grid
    teacher = ref["codes"].copy()
    teacher[2, 5] = teacher[2, 5] + (1 if teacher[2, 5] < 7 else -1)
    forced = O.gptq_quantize(W, U, 3, block=16, teacher_codes=teacher)
    assert forced["codes"][2, 5] == ref["codes"][2, 5] != teacher[2, 5]
    assert np.array_equal(forced["Q"], O.dequant(teacher, forced["scale"], forced["zero"]))
    assert np.allclose(W - forced["Q"], forced["E"] @ U, rtol=1e-9, atol=1e-13)   # the identity holds for any codes
    # U given as float32 is widened exactly
    U32 = U.astype(np.float32)
    a = O.gptq_quantize(W, U32, 3, block=16)
    b = O.gptq_quantize(W, U32.astype(np.float64), 3, block=16)
    assert np.array_equal(a["codes"], b["codes"]) and np.array_equal(a["E"], b["E"])


# ------------------------------------------------------------------ consumers of the packed format

def test_dequantize_and_matvec_by_hand():
    # the 3-bit words of test_pack_hand_computed_words: codes 1 2 3 4 5 6 7 0 1 2 7 (the last one straddles the words)
    words = np.array([[0xD11F58D1, 0x1]], dtype=np.uint32)
    Q = O.dequantize_packed(words, 11, 3, scale=[[0.5]], zero=[[3]])
    assert Q.tolist() == [[-1.0, -0.5, 0.0, 0.5, 1.0, 1.5, 2.0, -1.5, -1.0, -0.5, 2.0]]
    x = np.array([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11.0])
    # -1 - 1 + 0 + 2 + 5 + 9 + 14 - 12 - 9 - 5 + 22 = 24
    assert O.matvec_packed(words, 11, 3, [[0.5]], [[3]], 0, x).tolist() == [24.0]
    # two groups of 4 columns over 8 columns, 2-bit codes 3 0 1 2 | 3 0 1 2, scales 2 and 0.25, zeros 1 and 2
    w2 = np.array([[0x9393]], dtype=np.uint32)
    Qg = O.dequantize_packed(w2, 8, 2, scale=[[2.0, 0.25]], zero=[[1, 2]], group=4)
    assert Qg.tolist() == [[4.0, -2.0, 0.0, 2.0, 0.25, -0.5, -0.25, 0.0]]
    assert O.matvec_packed(w2, 8, 2, [[2.0, 0.25]], [[1, 2]], 4, np.ones(8)).tolist() == [3.5]


@pytest.mark.parametrize("bits,grid,group", [(3, "minmax", 0), (4, "minmax", 32), (2, "ternary", 8), (2, "minmax", 128)])
def test_packed_consumers_reproduce_algorithm_1_output(bits, grid, group):
    # what Alg. 1 calls Q is what the packed layer must stand for, bit for bit
    rng = np.random.default_rng(41 + bits)
    r, n = 9, 256
    W = rng.normal(size=(r, n)) * 0.02
    X = rng.normal(size=(n, 4 * n))
    U = O.hinv_cholesky_upper(O.damp(O.hessian(X)))
    out = O.gptq_quantize(W, U, bits, grid, 128, group)
    words = O.pack_codes(out["codes"], bits)
    Q = O.dequantize_packed(words, n, bits, out["scale"], out["zero"], group)
    assert np.array_equal(Q, out["Q"])
    x = rng.normal(size=n)
    y = O.matvec_packed(words, n, bits, out["scale"], out["zero"], group, x)
    loops = np.array([sum(out["Q"][i, k] * x[k] for k in range(n)) for i in range(r)])
    assert np.allclose(y, loops, rtol=1e-12, atol=1e-15)
    # closed form: equal codes c, one scale s, zero z  =>  y = s (c - z) sum(x)
    c = np.full((2, 70), 5 % (1 << bits))
    yc = O.matvec_packed(O.pack_codes(c, bits), 70, bits, [[0.5], [2.0]], [[1], [0]], 0, x[:70])
    assert np.allclose(yc, [0.5 * (c[0, 0] - 1) * x[:70].sum(), 2.0 * c[0, 0] * x[:70].sum()], rtol=1e-12)
