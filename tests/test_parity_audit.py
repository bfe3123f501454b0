"""The near-tie audit used by the GPU parity tests (tests/parity_util.py), exercised on the CPU with stand-ins
for a device result: it must accept a different arithmetic (ties flip and cascade) and reject planted mistakes."""
import numpy as np
import pytest

from oracle import gptq_oracle as O
from parity_util import audit_alg1, tie_distance


def _case(seed=3, r=48, n=256):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, 4 * n)) * np.exp(0.5 * rng.normal(size=(n, 1))) + 0.3 * rng.normal(size=(1, 4 * n))
    W = (rng.normal(size=(r, n)) * 0.02).astype(np.float16).astype(np.float64)
    Hd = O.damp(O.hessian(X))
    U = O.hinv_cholesky_upper(Hd).astype(np.float32).astype(np.float64)
    return W, U


@pytest.mark.parametrize("group,grid,bits", [(0, "minmax", 3), (64, "minmax", 2), (128, "ternary", 2)])
def test_audit_accepts_another_arithmetic(group, grid, bits):
    W, U = _case()
    quiet = lambda *_: None
    # a float32-decision run audited against float64 decisions, and the other way round
    a = O.gptq_quantize(W, U, bits, grid, 128, group, decision_dtype=np.float32)
    audit_alg1(W, U, bits, grid, 128, group, a["codes"], a["zero"], a["scale"], np.float64, say=quiet)
    # weights perturbed by 2e-5 of a grid step: decisions next to a tie flip and the flips cascade along their rows
    rng = np.random.default_rng(9)
    scale0 = O.grid_params(W, bits, grid)[0][:, None]
    b = O.gptq_quantize(W + 2e-5 * scale0 * rng.uniform(-1, 1, size=W.shape), U, bits, grid, 128, group)
    got = audit_alg1(W, U, bits, grid, 128, group, b["codes"], b["zero"], b["scale"], np.float64, say=quiet, scale_rtol=1e-4)
    assert got["max_tie_dist"] <= 1e-3


def test_audit_rejects_planted_mistakes():
    W, U = _case()
    quiet = lambda *_: None
    good = O.gptq_quantize(W, U, 3)
    # (1) one code moved by a step at a decision far from any tie, later columns untouched
    far = np.argwhere(tie_distance(good["frac"]) > 0.3)
    i, j = far[len(far) // 2]
    codes = good["codes"].copy()
    codes[i, j] += 1 if codes[i, j] < 7 else -1
    with pytest.raises(AssertionError):
        audit_alg1(W, U, 3, "minmax", 128, 0, codes, good["zero"], good["scale"], np.float64, say=quiet)
    # (2) an update that reads a wrong element of U: the run with U[5, 9] dropped differs at ordinary decisions
    Ubad = U.copy()
    Ubad[5, 9:40] = 0.0
    bad = O.gptq_quantize(W, Ubad, 3)
    assert (bad["codes"] != good["codes"]).any()
    with pytest.raises(AssertionError):
        audit_alg1(W, U, 3, "minmax", 128, 0, bad["codes"], bad["zero"], bad["scale"], np.float64, say=quiet)
    # (3) truncation instead of round-to-nearest
    trunc = np.clip(np.floor(good["frac"]).astype(np.int64) + good["zero"], 0, 7)
    with pytest.raises(AssertionError):
        audit_alg1(W, U, 3, "minmax", 128, 0, trunc, good["zero"], good["scale"], np.float64, say=quiet)


def test_audit_zero_point_ties():
    W, U = _case(seed=5, r=16, n=128)
    quiet = lambda *_: None
    # row 3: lo = -1.5 s, hi = +1.5 s at 2 bits, so -lo/scale = 1.5 exactly: rint gives 2; an arithmetic that sees
    # 1.4999999 gives 1 and clamps at the other end of the range
    W[3] = np.clip(W[3], -0.03, 0.03)
    W[3, 10], W[3, 20] = -0.046875, 0.046875
    good = O.gptq_quantize(W, U, 2)
    assert good["zero"][3, 0] == 2 and good["zero_real"][3, 0] == 1.5
    Wn = W.copy()
    Wn[3, 10] *= (1 - 1e-9)
    other = O.gptq_quantize(Wn, U, 2)
    assert other["zero"][3, 0] == 1
    audit_alg1(W, U, 2, "minmax", 128, 0, other["codes"], other["zero"], other["scale"], np.float64, say=quiet)
    # a zero point that is off by one where -lo/scale is nowhere near a half-integer is a mistake
    far = int(np.argmax(np.abs(np.abs(good["zero_real"][:, 0] % 1.0 - 0.5) - 0.5) < 0.2))
    zbad = good["zero"].copy()
    zbad[far, 0] += 1
    cbad = np.clip(good["codes"] + (np.arange(16) == far)[:, None], 0, 3)
    with pytest.raises(AssertionError):
        audit_alg1(W, U, 2, "minmax", 128, 0, cbad, zbad, good["scale"], np.float64, say=quiet)
